// C ABI of the NVFP4 library (see include/nvfp4.h): argument validation and
// dispatch only; every step of the path runs in the kernels.
#include "nvfp4.h"
#include "nvfp4_internal.h"

// Scratch of nvfp4_quantize_static, the entry point for callers that cannot allocate: the quantizer's workspace (the
// amax pass's per-workgroup maxima and their fold) in device memory that belongs to the library's code object.  Every
// GPU the library runs on holds its own copy of this array, at its own address, until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress -- never a device address.
static __device__ __align__(256) unsigned char scratch[NVFP4_STATIC_SCRATCH_BYTES];   // size: include/nvfp4.h

namespace nvfp4 {

namespace {

void host_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c[4] = {ctr[0], ctr[1], ctr[2], ctr[3]};
  uint32_t k[2] = {key[0], key[1]};
  for (int round = 0; round < 10; ++round) {
    const uint64_t lo = 0xD2511F53ull * c[0], hi = 0xCD9E8D57ull * c[2];
    const uint32_t t0 = static_cast<uint32_t>(hi >> 32) ^ c[1] ^ k[0];
    const uint32_t t2 = static_cast<uint32_t>(lo >> 32) ^ c[3] ^ k[1];
    c[1] = static_cast<uint32_t>(hi);
    c[3] = static_cast<uint32_t>(lo);
    c[0] = t0;
    c[2] = t2;
    k[0] += 0x9E3779B9u;
    k[1] += 0xBB67AE85u;
  }
  for (int i = 0; i < 4; ++i) out[i] = c[i];
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Rotation size asked for by nvfp4_quantize's rht_on_col: 0 none, 1 the format's own (16; 32 for MXFP4), or the
// size itself.  Returns -1 for a size the format does not have.
int rotation_size(int rht_on_col, bool mx) {
  if (rht_on_col == 0) return 0;
  if (rht_on_col == 1) return mx ? 32 : 16;
  if (mx) return rht_on_col == 32 ? 32 : -1;
  return (rht_on_col == 2 || rht_on_col == 4 || rht_on_col == 16 || rht_on_col == 32 || rht_on_col == 128) ? rht_on_col : -1;
}

// The sign diagonal in the forms the kernels take (QuantizeArgs): all its bits, and for sizes up to 32 one word
// (sizes below 16 repeated over the low 16 bits, since those kernels walk 16 rows at a time).
void fill_signs(uint64_t seed, int d, uint32_t* mask, uint32_t words[4]) {
  words[0] = words[1] = words[2] = words[3] = 0u;
  *mask = 0u;
  if (d == 0) return;
  host_rht_sign_words(seed, words);
  if (d >= 32) {
    *mask = words[0];
  } else {
    const uint32_t bits = words[0] & ((1u << d) - 1u);
    for (int i = 0; i < 16; i += d) *mask |= bits << i;
    if (d == 16) *mask = bits;
  }
}


}  // namespace

uint32_t host_rht_sign_mask32(uint64_t seed) {
  const uint32_t ctr[4] = {0u, 0u, 0u, 0xFFFFFFFFu};
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  uint32_t out[4];
  host_philox4x32_10(ctr, key, out);
  return out[0];
}

uint32_t host_rht_sign_mask(uint64_t seed) { return host_rht_sign_mask32(seed) & 0xFFFFu; }

void host_rht_sign_words(uint64_t seed, uint32_t words[4]) {
  const uint32_t ctr[4] = {0u, 0u, 0u, 0xFFFFFFFFu};
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  host_philox4x32_10(ctr, key, words);
}

}  // namespace nvfp4

using namespace nvfp4;

extern "C" {

int nvfp4_version(void) { return 100; }

const char* nvfp4_status_string(int status) {
  switch (status) {
    case NVFP4_OK: return "ok";
    case NVFP4_ERR_INVALID_ARG: return "invalid argument (null pointer, unknown enum, misaligned pointer)";
    case NVFP4_ERR_BAD_SHAPE: return "bad shape (rows/cols must be positive multiples of 16; leading dimension too small or misaligned)";
    case NVFP4_ERR_MISSING_COPY: return "the quantized tensor lacks the copy this operation needs";
    case NVFP4_ERR_MISMATCH: return "operands disagree (contraction length, rotation size or rotation seed)";
    case NVFP4_ERR_HIP: return "HIP runtime error";
    case NVFP4_ERR_WORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
  }
}

uint32_t nvfp4_rht_sign_mask(uint64_t rht_seed) { return host_rht_sign_mask(rht_seed); }

int nvfp4_quantized_sizes(int64_t rows, int64_t cols, size_t* codes_bytes, size_t* scales_bytes,
                          size_t* workspace_bytes) {
  if (rows <= 0 || cols <= 0 || rows % 16 || cols % 16) return NVFP4_ERR_BAD_SHAPE;
  if (codes_bytes) *codes_bytes = static_cast<size_t>(rows) * static_cast<size_t>(cols) / 2;
  if (scales_bytes) *scales_bytes = static_cast<size_t>(rows) * static_cast<size_t>(cols) / 16;
  if (workspace_bytes) *workspace_bytes = quantize_workspace_bytes(rows, cols);
  return NVFP4_OK;
}

namespace {

// A validated nvfp4_quantize call: kernel arguments plus the descriptor as it will read afterwards.
struct QuantPlan {
  QuantizeArgs a;
  nvfp4_qtensor desc;
};

// amax_given: pass 2 only; `workspace` then is the caller's two amax words and no workspace size applies.
int plan_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, int layout_mask, int block_dim, int rounding,
                  int rht_on_col, uint64_t rht_seed, uint64_t sr_seed, const nvfp4_qtensor* out, void* workspace,
                  size_t workspace_bytes, QuantPlan* p, bool amax_given = false) {
  if (!x || !out) return NVFP4_ERR_INVALID_ARG;
  if (layout_mask <= 0 || (layout_mask & ~(NVFP4_LAYOUT_ROW | NVFP4_LAYOUT_COL | NVFP4_LAYOUT_ROW_RHT | NVFP4_LAYOUT_ROW_SCALES)))
    return NVFP4_ERR_INVALID_ARG;
  const bool row_rht = layout_mask & NVFP4_LAYOUT_ROW_RHT;
  const bool scale_per_row = layout_mask & NVFP4_LAYOUT_ROW_SCALES;
  layout_mask &= NVFP4_LAYOUT_ROW | NVFP4_LAYOUT_COL;
  if (layout_mask == 0) return NVFP4_ERR_INVALID_ARG;
  if (block_dim != NVFP4_BLOCK_1x16 && block_dim != NVFP4_BLOCK_16x16 && block_dim != NVFP4_BLOCK_MX32)
    return NVFP4_ERR_INVALID_ARG;
  if (rounding != NVFP4_ROUND_RNE && rounding != NVFP4_ROUND_SR) return NVFP4_ERR_INVALID_ARG;
  const bool want_row = layout_mask & NVFP4_LAYOUT_ROW, want_col = layout_mask & NVFP4_LAYOUT_COL;
  const bool mx = block_dim == NVFP4_BLOCK_MX32;
  const int rht_dim = rotation_size(rht_on_col, mx);
  if (rht_dim < 0 || (rht_dim && (block_dim == NVFP4_BLOCK_16x16 || !want_col))) return NVFP4_ERR_INVALID_ARG;
  // A rotated row copy: NVFP4 1x16 blocks, the 16-point rotation only, both passes in this call.
  if (row_rht && (!want_row || block_dim != NVFP4_BLOCK_1x16 || (rht_dim && rht_dim != 16) || amax_given))
    return NVFP4_ERR_INVALID_ARG;
  // One tensor-level scale per row of each copy: NVFP4 1x16 blocks (a 16x16 weight tile's scale must serve both
  // orientations, Sec. 4.3), the recipe's rotation or none, both passes in this call.
  if (scale_per_row && (block_dim != NVFP4_BLOCK_1x16 || row_rht || (rht_dim && rht_dim != 16) || amax_given))
    return NVFP4_ERR_INVALID_ARG;
  if (rows <= 0 || cols <= 0 || rows % 16 || cols % 16 || ld < cols || ld % 8) return NVFP4_ERR_BAD_SHAPE;
  if (rht_dim && rows % rht_dim) return NVFP4_ERR_BAD_SHAPE;   // whole rotation groups along the rows
  if (mx && (rows % 32 || cols % 32)) return NVFP4_ERR_BAD_SHAPE;
  if (!aligned(x, 16)) return NVFP4_ERR_INVALID_ARG;
  if (want_row && (!out->row_codes || !out->row_scales || !out->row_tensor_scale)) return NVFP4_ERR_INVALID_ARG;
  if (want_col && (!out->col_codes || !out->col_scales || !out->col_tensor_scale)) return NVFP4_ERR_INVALID_ARG;
  if (scale_per_row && ((want_row && !aligned(out->row_tensor_scale, 16)) || (want_col && !aligned(out->col_tensor_scale, 16))))
    return NVFP4_ERR_INVALID_ARG;   // the GEMM reads the scale vectors in 16-byte pieces
  if (want_row && (!aligned(out->row_codes, 16) || !aligned(out->row_scales, 16))) return NVFP4_ERR_INVALID_ARG;
  if (want_col && (!aligned(out->col_codes, 16) || !aligned(out->col_scales, 16))) return NVFP4_ERR_INVALID_ARG;
  // the MXFP4 mode is a single pass and needs no workspace
  if (amax_given) {
    if (mx || !workspace || !aligned(workspace, 4)) return NVFP4_ERR_INVALID_ARG;
  } else if (!mx && (!workspace || workspace_bytes < quantize_workspace_bytes(rows, cols) || !aligned(workspace, 16))) {
    return NVFP4_ERR_WORKSPACE;
  }

  QuantizeArgs& a = p->a;
  a.x = x;
  a.rows = rows;
  a.cols = cols;
  a.ld = ld;
  a.want_row = want_row;
  a.want_col = want_col;
  a.rht = rht_dim != 0;
  a.rht_dim = rht_dim;
  a.sr = rounding == NVFP4_ROUND_SR;
  a.block2d = block_dim == NVFP4_BLOCK_16x16;
  a.row_rht = row_rht;
  a.scale_per_row = scale_per_row;
  fill_signs(rht_seed, row_rht ? 16 : rht_dim, &a.sign_mask, a.sign_words);
  a.key0 = static_cast<uint32_t>(sr_seed);
  a.key1 = static_cast<uint32_t>(sr_seed >> 32);
  a.ws = static_cast<uint32_t*>(workspace);
  a.do_amax = !amax_given;
  a.row_codes = static_cast<uint8_t*>(out->row_codes);
  a.row_scales = static_cast<uint8_t*>(out->row_scales);
  a.row_ts = out->row_tensor_scale;
  a.col_codes = static_cast<uint8_t*>(out->col_codes);
  a.col_scales = static_cast<uint8_t*>(out->col_scales);
  a.col_ts = out->col_tensor_scale;

  p->desc = *out;
  p->desc.rows = rows;
  p->desc.cols = cols;
  p->desc.layout_mask = layout_mask;
  p->desc.block_dim = block_dim;
  p->desc.rounding = rounding;
  p->desc.col_has_rht = rht_dim;
  p->desc.row_has_rht = row_rht ? 16 : 0;
  p->desc.scale_per_row = scale_per_row ? 1 : 0;
  p->desc.row_fp16 = nullptr;   // decoded copies of the previous contents are stale
  p->desc.col_fp16 = nullptr;
  p->desc.rht_seed = (a.rht || row_rht) ? rht_seed : 0;
  return NVFP4_OK;
}

}  // namespace

int nvfp4_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int rht_on_col, uint64_t rht_seed, float* amax_out,
               void* workspace, size_t workspace_bytes, nvfp4_stream_t stream) {
  if (!x || !amax_out || !aligned(x, 16) || !aligned(amax_out, 4)) return NVFP4_ERR_INVALID_ARG;
  const int rht_dim = rotation_size(rht_on_col, false);
  if (rht_dim < 0) return NVFP4_ERR_INVALID_ARG;
  if (rows <= 0 || cols <= 0 || rows % 16 || cols % 16 || ld < cols || ld % 8) return NVFP4_ERR_BAD_SHAPE;
  if (rht_dim && rows % rht_dim) return NVFP4_ERR_BAD_SHAPE;
  if (!workspace || workspace_bytes < quantize_workspace_bytes(rows, cols) || !aligned(workspace, 16)) return NVFP4_ERR_WORKSPACE;
  QuantizeArgs a{};
  a.x = x;
  a.rows = rows;
  a.cols = cols;
  a.ld = ld;
  a.want_row = true;            // the amax of the tensor itself is always computed
  a.want_col = rht_dim != 0;    // that of the rotated tensor if a rotation is named
  a.rht = rht_dim != 0;
  a.rht_dim = rht_dim;
  fill_signs(rht_seed, rht_dim, &a.sign_mask, a.sign_words);
  a.ws = static_cast<uint32_t*>(workspace);
  a.do_amax = true;
  a.do_cast = false;
  a.amax_copy = reinterpret_cast<uint32_t*>(amax_out);
  return launch_quantize(a, static_cast<hipStream_t>(stream)) == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_quantize_with_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int layout_mask, int block_dim,
                             int rounding, int rht_on_col, uint64_t rht_seed, uint64_t sr_seed, const float* amax_in,
                             nvfp4_qtensor* out, nvfp4_stream_t stream) {
  QuantPlan p;
  const int rc = plan_quantize(x, rows, cols, ld, layout_mask, block_dim, rounding, rht_on_col, rht_seed, sr_seed, out,
                               const_cast<float*>(amax_in), 0, &p, true);
  if (rc != NVFP4_OK) return rc;
  if (launch_quantize(p.a, static_cast<hipStream_t>(stream)) != hipSuccess) return NVFP4_ERR_HIP;
  *out = p.desc;
  return NVFP4_OK;
}

int nvfp4_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, int layout_mask, int block_dim,
                   int rounding, int rht_on_col, uint64_t rht_seed, uint64_t sr_seed, nvfp4_qtensor* out,
                   void* workspace, size_t workspace_bytes, nvfp4_stream_t stream) {
  QuantPlan p;
  const int rc = plan_quantize(x, rows, cols, ld, layout_mask, block_dim, rounding, rht_on_col, rht_seed, sr_seed, out,
                               workspace, workspace_bytes, &p);
  if (rc != NVFP4_OK) return rc;
  const hipError_t e = block_dim == NVFP4_BLOCK_MX32 ? launch_quantize_mx(p.a, static_cast<hipStream_t>(stream))
                                                     : launch_quantize(p.a, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return NVFP4_ERR_HIP;
  *out = p.desc;
  return NVFP4_OK;
}

namespace {

// Device address of `scratch` on the current device, looked up once per device (with that device current) and kept.
constexpr int kMaxDevices = 64;
std::atomic<void*> scratch_address[kMaxDevices];

int static_scratch(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return NVFP4_ERR_HIP;
  void* p = scratch_address[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return NVFP4_ERR_HIP;
    scratch_address[dev].store(p, std::memory_order_release);   // two threads racing here store the same address
  }
  *ptr = p;
  return NVFP4_OK;
}

}  // namespace

int nvfp4_quantize_static(const void* x, int64_t rows, int64_t cols, int64_t ld, int layout_mask, int block_dim,
                          int rounding, int rht_on_col, uint64_t rht_seed, uint64_t sr_seed, nvfp4_qtensor* out,
                          nvfp4_stream_t stream) {
  const bool mx = block_dim == NVFP4_BLOCK_MX32;
  // the size limit first: it needs no GPU and no other argument
  if (!mx && rows > 0 && cols > 0 && rows % 16 == 0 && cols % 16 == 0 &&
      quantize_workspace_bytes(rows, cols) > NVFP4_STATIC_SCRATCH_BYTES)
    return NVFP4_ERR_WORKSPACE;
  // every other check with a stand-in for the workspace address, so that a bad call is refused before any HIP call
  QuantPlan p;
  void* const stand_in = reinterpret_cast<void*>(uintptr_t{256});
  const int rc = plan_quantize(x, rows, cols, ld, layout_mask, block_dim, rounding, rht_on_col, rht_seed, sr_seed, out,
                               stand_in, NVFP4_STATIC_SCRATCH_BYTES, &p);
  if (rc != NVFP4_OK) return rc;
  if (!mx) {
    void* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs != NVFP4_OK) return rs;
    p.a.ws = static_cast<uint32_t*>(ws);   // the kernels take the looked-up address, as they take a caller's workspace
  }
  const hipError_t e = mx ? launch_quantize_mx(p.a, static_cast<hipStream_t>(stream)) : launch_quantize(p.a, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return NVFP4_ERR_HIP;
  *out = p.desc;
  return NVFP4_OK;
}

static int pick_operand(const nvfp4_qtensor* q, bool col_copy, Operand* op, int64_t* K) {
  if (col_copy) {
    if (!(q->layout_mask & NVFP4_LAYOUT_COL) || !q->col_codes || !q->col_scales || !q->col_tensor_scale)
      return NVFP4_ERR_MISSING_COPY;
    op->codes = static_cast<const uint8_t*>(q->col_codes);
    op->scales = static_cast<const uint8_t*>(q->col_scales);
    op->ts = q->col_tensor_scale;
    op->outer = q->cols;
    op->fp16 = q->col_fp16;
    op->ts_per_row = q->scale_per_row ? 1 : 0;
    *K = q->rows;
  } else {
    if (!(q->layout_mask & NVFP4_LAYOUT_ROW) || !q->row_codes || !q->row_scales || !q->row_tensor_scale)
      return NVFP4_ERR_MISSING_COPY;
    op->codes = static_cast<const uint8_t*>(q->row_codes);
    op->scales = static_cast<const uint8_t*>(q->row_scales);
    op->ts = q->row_tensor_scale;
    op->outer = q->rows;
    op->fp16 = q->row_fp16;
    op->ts_per_row = q->scale_per_row ? 1 : 0;
    *K = q->cols;
  }
  return NVFP4_OK;
}

int nvfp4_predecode(nvfp4_qtensor* q, int which_copy, void* fp16_out, size_t fp16_bytes, nvfp4_stream_t stream) {
  if (!q || !fp16_out || !aligned(fp16_out, 16)) return NVFP4_ERR_INVALID_ARG;
  if (which_copy != NVFP4_COPY_ROW && which_copy != NVFP4_COPY_COL) return NVFP4_ERR_INVALID_ARG;
  if (q->block_dim == NVFP4_BLOCK_MX32) return NVFP4_ERR_INVALID_ARG;   // MXFP4 operands feed the matrix pipe as they are
  Operand op;
  int64_t K = 0;
  const int rc = pick_operand(q, which_copy == NVFP4_COPY_COL, &op, &K);
  if (rc != NVFP4_OK) return rc;
  if (K <= 0 || K % 64 || op.outer <= 0) return NVFP4_ERR_BAD_SHAPE;   // the decoded layout is made of 8-row x 64-k pieces
  if (!aligned(op.codes, 16) || !aligned(op.scales, 4)) return NVFP4_ERR_INVALID_ARG;
  if (fp16_bytes < static_cast<size_t>(op.outer) * static_cast<size_t>(K) * 2) return NVFP4_ERR_WORKSPACE;
  if (launch_predecode(op, K, fp16_out, static_cast<hipStream_t>(stream)) != hipSuccess) return NVFP4_ERR_HIP;
  if (which_copy == NVFP4_COPY_COL) q->col_fp16 = fp16_out; else q->row_fp16 = fp16_out;
  return NVFP4_OK;
}

int nvfp4_gemm_workspace_bytes(int64_t m, int64_t n, int64_t k, size_t* workspace_bytes) {
  if (m <= 0 || n <= 0 || k <= 0 || m % 16 || n % 16 || k % 16) return NVFP4_ERR_BAD_SHAPE;
  if (!workspace_bytes) return NVFP4_ERR_INVALID_ARG;
  *workspace_bytes = gemm_workspace_bytes(m, n, k);
  return NVFP4_OK;
}

static int plan_gemm(const nvfp4_qtensor* a, const nvfp4_qtensor* b, int op, void* d, int out_dtype, int64_t ldd,
                     void* workspace, size_t workspace_bytes, GemmArgs* gp) {
  if (!a || !b || !d) return NVFP4_ERR_INVALID_ARG;
  if (out_dtype != NVFP4_OUT_F32 && out_dtype != NVFP4_OUT_BF16 && out_dtype != NVFP4_OUT_F32_ACCUMULATE)
    return NVFP4_ERR_INVALID_ARG;
  bool a_col, b_col;
  switch (op) {
    case NVFP4_OP_FPROP: a_col = false; b_col = true; break;
    case NVFP4_OP_DGRAD: a_col = false; b_col = false; break;
    case NVFP4_OP_WGRAD: a_col = true; b_col = true; break;
    default: return NVFP4_ERR_INVALID_ARG;
  }
  GemmArgs& g = *gp;
  int64_t ka = 0, kb = 0;
  int rc = pick_operand(a, a_col, &g.a, &ka);
  if (rc != NVFP4_OK) return rc;
  rc = pick_operand(b, b_col, &g.b, &kb);
  if (rc != NVFP4_OK) return rc;
  if (ka != kb) return NVFP4_ERR_MISMATCH;
  // Both operands in the same format: NVFP4 (E4M3 scale per 16) or MXFP4 (UE8M0 scale per 32).
  const bool a_mx = a->block_dim == NVFP4_BLOCK_MX32, b_mx = b->block_dim == NVFP4_BLOCK_MX32;
  if (a_mx != b_mx) return NVFP4_ERR_MISMATCH;
  if (a_mx && (a->scale_per_row || b->scale_per_row)) return NVFP4_ERR_INVALID_ARG;   // MXFP4 has no tensor-level scale
  if ((g.a.ts_per_row && !aligned(g.a.ts, 16)) || (g.b.ts_per_row && !aligned(g.b.ts, 16))) return NVFP4_ERR_INVALID_ARG;
  if (a_mx && (ka % 128 || g.a.outer % 32 || g.b.outer % 32)) return NVFP4_ERR_BAD_SHAPE;   // one scaled MFMA is 128 deep
  if (a_mx && (!aligned(g.a.codes, 16) || !aligned(g.b.codes, 16) || !aligned(g.a.scales, 4) || !aligned(g.b.scales, 4)))
    return NVFP4_ERR_INVALID_ARG;
  g.mx = a_mx;
  // Rotated operands only make sense in pairs that rotate the same way (App. C).
  const int a_rot = a_col ? a->col_has_rht : a->row_has_rht, b_rot = b_col ? b->col_has_rht : b->row_has_rht;   // rotation sizes
  if (a_rot != b_rot || (a_rot && a->rht_seed != b->rht_seed)) return NVFP4_ERR_MISMATCH;
  if (ka <= 0 || ka % 16 || g.a.outer <= 0 || g.b.outer <= 0) return NVFP4_ERR_BAD_SHAPE;
  if (ldd < g.b.outer || ldd % (out_dtype == NVFP4_OUT_BF16 ? 8 : 4)) return NVFP4_ERR_BAD_SHAPE;   // 16-byte output pieces
  if (!aligned(d, 16) || !aligned(g.a.codes, 8) || !aligned(g.b.codes, 8)) return NVFP4_ERR_INVALID_ARG;
  g.K = ka;
  g.d = d;
  g.ldd = ldd;
  g.out_bf16 = out_dtype == NVFP4_OUT_BF16;
  g.accumulate = out_dtype == NVFP4_OUT_F32_ACCUMULATE;
  g.workspace = workspace;
  g.workspace_bytes = workspace ? workspace_bytes : 0;
  return NVFP4_OK;
}

int nvfp4_gemm(const nvfp4_qtensor* a, const nvfp4_qtensor* b, int op, void* d, int out_dtype, int64_t ldd,
               void* workspace, size_t workspace_bytes, nvfp4_stream_t stream) {
  GemmArgs g;
  const int rc = plan_gemm(a, b, op, d, out_dtype, ldd, workspace, workspace_bytes, &g);
  if (rc != NVFP4_OK) return rc;
  const hipError_t e = g.mx ? launch_gemm_mx(g, static_cast<hipStream_t>(stream)) : launch_gemm(g, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

// ---------------------------------------------------------------- one linear layer (Sec. 4.1, Fig. 3)

int nvfp4_linear_workspace_bytes(int64_t tokens, int64_t d_in, int64_t d_out, size_t* workspace_bytes) {
  if (tokens <= 0 || d_in <= 0 || d_out <= 0 || tokens % 16 || d_in % 16 || d_out % 16) return NVFP4_ERR_BAD_SHAPE;
  if (!workspace_bytes) return NVFP4_ERR_INVALID_ARG;
  size_t need = quantize_workspace_bytes(tokens, d_in);
  const size_t parts[4] = {quantize_workspace_bytes(tokens, d_out), gemm_workspace_bytes(tokens, d_out, d_in),
                           gemm_workspace_bytes(tokens, d_in, d_out), gemm_workspace_bytes(d_in, d_out, tokens)};
  for (size_t b : parts) need = b > need ? b : need;
  *workspace_bytes = need;
  return NVFP4_OK;
}

int nvfp4_linear_forward(const void* x, int64_t tokens, int64_t d_in, int64_t ldx, const nvfp4_qtensor* qw,
                         int keep_for_backward, uint64_t rht_seed, nvfp4_qtensor* qx, void* y, int out_dtype,
                         int64_t ldy, void* workspace, size_t workspace_bytes, nvfp4_stream_t stream) {
  if (!qw || !qx || !y) return NVFP4_ERR_INVALID_ARG;
  QuantPlan px;
  const int layouts = keep_for_backward ? (NVFP4_LAYOUT_ROW | NVFP4_LAYOUT_COL) : NVFP4_LAYOUT_ROW;
  int rc = plan_quantize(x, tokens, d_in, ldx, layouts, NVFP4_BLOCK_1x16, NVFP4_ROUND_RNE, keep_for_backward ? 1 : 0,
                         rht_seed, 0, qx, workspace, workspace_bytes, &px);
  if (rc != NVFP4_OK) return rc;
  GemmArgs g;
  rc = plan_gemm(&px.desc, qw, NVFP4_OP_FPROP, y, out_dtype, ldy, workspace, workspace_bytes, &g);
  if (rc != NVFP4_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (launch_quantize(px.a, s) != hipSuccess) return NVFP4_ERR_HIP;
  *qx = px.desc;
  return launch_gemm(g, s) == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_linear_backward(const void* dy, int64_t tokens, int64_t d_out, int64_t lddy, const nvfp4_qtensor* qx,
                          const nvfp4_qtensor* qw, uint64_t sr_seed, nvfp4_qtensor* qdy, void* dx, int dx_dtype,
                          int64_t lddx, float* dw, int64_t lddw, int accumulate_dw, void* workspace,
                          size_t workspace_bytes, nvfp4_stream_t stream) {
  if (!qx || !qw || !qdy || !dx || !dw) return NVFP4_ERR_INVALID_ARG;
  if (dx_dtype != NVFP4_OUT_F32 && dx_dtype != NVFP4_OUT_BF16) return NVFP4_ERR_INVALID_ARG;
  if (!(qx->layout_mask & NVFP4_LAYOUT_COL) || !qx->col_has_rht) return NVFP4_ERR_MISSING_COPY;
  QuantPlan pdy;
  int rc = plan_quantize(dy, tokens, d_out, lddy, NVFP4_LAYOUT_ROW | NVFP4_LAYOUT_COL, NVFP4_BLOCK_1x16,
                         NVFP4_ROUND_SR, qx->col_has_rht, qx->rht_seed, sr_seed, qdy, workspace, workspace_bytes, &pdy);
  if (rc != NVFP4_OK) return rc;
  GemmArgs dgrad, wgrad;
  rc = plan_gemm(&pdy.desc, qw, NVFP4_OP_DGRAD, dx, dx_dtype, lddx, workspace, workspace_bytes, &dgrad);
  if (rc != NVFP4_OK) return rc;
  rc = plan_gemm(qx, &pdy.desc, NVFP4_OP_WGRAD, dw, accumulate_dw ? NVFP4_OUT_F32_ACCUMULATE : NVFP4_OUT_F32, lddw,
                 workspace, workspace_bytes, &wgrad);
  if (rc != NVFP4_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (launch_quantize(pdy.a, s) != hipSuccess) return NVFP4_ERR_HIP;
  *qdy = pdy.desc;
  if (launch_gemm(dgrad, s) != hipSuccess) return NVFP4_ERR_HIP;
  return launch_gemm(wgrad, s) == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_dequantize(const nvfp4_qtensor* q, int which_copy, int undo_rht, void* out, int out_dtype,
                     int64_t ld_out, nvfp4_stream_t stream) {
  if (!q || !out) return NVFP4_ERR_INVALID_ARG;
  if (which_copy != NVFP4_COPY_ROW && which_copy != NVFP4_COPY_COL) return NVFP4_ERR_INVALID_ARG;
  if (out_dtype != NVFP4_OUT_F32 && out_dtype != NVFP4_OUT_BF16) return NVFP4_ERR_INVALID_ARG;
  DequantArgs d;
  int rc = pick_operand(q, which_copy == NVFP4_COPY_COL, &d.q, &d.K);
  if (rc != NVFP4_OK) return rc;
  const int copy_rht = which_copy == NVFP4_COPY_COL ? q->col_has_rht : q->row_has_rht;
  if (undo_rht && !copy_rht) return NVFP4_ERR_MISMATCH;
  const bool mx = q->block_dim == NVFP4_BLOCK_MX32;
  if (d.K <= 0 || d.K % (mx ? 32 : 16) || ld_out < d.K || ld_out % 8) return NVFP4_ERR_BAD_SHAPE;
  if (!aligned(out, 16) || !aligned(d.q.codes, mx ? 16 : 8)) return NVFP4_ERR_INVALID_ARG;
  d.undo_rht = undo_rht != 0;
  d.rht_dim = d.undo_rht ? copy_rht : 0;
  if (d.undo_rht && (rotation_size(d.rht_dim, mx) != d.rht_dim || d.rht_dim == 1 || d.K % d.rht_dim)) return NVFP4_ERR_MISMATCH;
  fill_signs(q->rht_seed, d.rht_dim, &d.sign_mask, d.sign_words);
  d.out = out;
  d.ld_out = ld_out;
  d.out_bf16 = out_dtype == NVFP4_OUT_BF16;
  const hipError_t e = mx ? launch_dequantize_mx(d, static_cast<hipStream_t>(stream)) : launch_dequantize(d, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_selftest_conversions(uint64_t* mismatches, nvfp4_stream_t stream) {
  if (!mismatches || !aligned(mismatches, 8)) return NVFP4_ERR_INVALID_ARG;
  return run_selftest(mismatches, static_cast<hipStream_t>(stream)) == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

}  // extern "C"
