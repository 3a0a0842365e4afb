// MXFP4 quantizer for gfx950: the paper's comparison format (Sec. 2: E2M1
// elements, blocks of 32, one UE8M0 power-of-two scale per block; App. B.4:
// the scale is amax_b / 6 rounded up to a power of two so nothing saturates;
// Sec. 5: a 32-point random Hadamard rotation on the Wgrad operands).
//
// There is no tensor-level scale, so one pass over the tensor is enough.
// Work decomposition: a lane owns 32 rows x 8 columns (thirty-two 128-bit loads);
// a wavefront owns 32 rows x 512 columns; a 256-thread workgroup 128 rows x 512
// columns.  A row-copy block (32 columns of one row) is four neighbouring lanes
// (two cross-lane maxima); a col-copy block (32 rows of one column) and the whole
// 32-point butterfly live in one lane's registers.  Row codes leave as one dword
// per lane and row; everything else is staged in LDS and written back as
// contiguous pieces (64 bytes of codes per column per workgroup).
//
// Random draws: the row copy uses the NVFP4 draws (counter (j / 8, i, 0, 0)); the
// col copy draws its own, counter (i / 8, j, 1, 0), word (i % 8) / 2, low half for
// even i, so that eight consecutive rows of a column come from one Philox call.
#include "nvfp4_internal.h"
#include "nvfp4_device.h"

namespace nvfp4 {

namespace {

constexpr int kThreads = 256;
constexpr int kWaveCols = 512;
constexpr int kRowsPerWave = 32;
constexpr int kRowsPerBlock = 128;
constexpr int kSlot = 65;   // lanes per staging row, padded

// amax_b / 6 rounded up to a power of two 2^e, e clamped to [-127, 127] (App. B.4).
// Returns the stored byte e + 127 and the exact encode factor 2^-e.
__device__ __forceinline__ uint32_t ue8m0_scale(float amax_b, float& inv) {
  const uint32_t bits = __float_as_uint(div_by_6(amax_b));
  const int E = static_cast<int>(bits >> 23), M = static_cast<int>(bits & 0x7FFFFFu);
  int e;
  if (E > 0) e = E - 127 + (M != 0 ? 1 : 0);
  else e = M > 0x400000 ? -126 : -127;   // subnormal quotient (or zero)
  e = min(e, 127);
  inv = __uint_as_float(e == 127 ? 0x00400000u : static_cast<uint32_t>(127 - e) << 23);
  return static_cast<uint32_t>(e + 127);
}

// Eight values -> one dword of eight codes (value t in nibble t).
template <bool kSR>
__device__ __forceinline__ uint32_t encode8(const float v[8], const uint32_t draws_hi16[8]) {
  if (!kSR) {
    uint32_t d = 0;
    d = cvt_rne_pair<0>(d, v[0], v[1]);
    d = cvt_rne_pair<1>(d, v[2], v[3]);
    d = cvt_rne_pair<2>(d, v[4], v[5]);
    d = cvt_rne_pair<3>(d, v[6], v[7]);
    return d;
  } else {
    uint32_t e = 0u, o = 0u;
    cvt_sr_single_into<0>(e, v[0], draws_hi16[0]);
    cvt_sr_single_into<1>(e, v[2], draws_hi16[2]);
    cvt_sr_single_into<2>(e, v[4], draws_hi16[4]);
    cvt_sr_single_into<3>(e, v[6], draws_hi16[6]);
    cvt_sr_single_into<0>(o, v[1], draws_hi16[1]);
    cvt_sr_single_into<1>(o, v[3], draws_hi16[3]);
    cvt_sr_single_into<2>(o, v[5], draws_hi16[5]);
    cvt_sr_single_into<3>(o, v[7], draws_hi16[7]);
    return interleave_nibbles(e, o);
  }
}

// the eight 16-bit draws of one Philox call, each moved to the top half of a word
__device__ __forceinline__ void draws8(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t k0, uint32_t k1, uint32_t out[8]) {
  uint32_t w[4];
  philox4x32_10(c0, c1, c2, 0u, k0, k1, w);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    out[2 * t] = w[t] << 16;
    out[2 * t + 1] = w[t] & 0xFFFF0000u;
  }
}

__device__ __forceinline__ float elem(const uint4& q, int c) {
  const uint32_t w = (c < 2) ? q.x : (c < 4) ? q.y : (c < 6) ? q.z : q.w;
  return (c & 1) ? bf16_hi(w) : bf16_lo(w);
}

template <bool kRow, bool kCol, bool kRht, bool kSR>
__global__ __launch_bounds__(kThreads) void quantize_mx_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                               int64_t ld, uint32_t sign_mask, uint32_t key0, uint32_t key1,
                                                               uint8_t* __restrict__ row_codes, uint8_t* __restrict__ row_scales,
                                                               uint8_t* __restrict__ col_codes, uint8_t* __restrict__ col_scales) {
  __shared__ __attribute__((aligned(16))) uint8_t st_col_codes[8 * 4 * kSlot * 16];   // [column of the lane][wavefront][lane] x 16 bytes
  __shared__ uint8_t st_col_scales[8 * 4 * 64];                                       // [column of the lane][wavefront][lane]
  __shared__ __attribute__((aligned(16))) uint8_t st_row_scales[4 * kRowsPerWave * 16];   // [wavefront][row][16 blocks]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t colblk = static_cast<int64_t>(blockIdx.x) * kWaveCols;
  const int64_t col0 = colblk + lane * 8;
  const int64_t rowblk = static_cast<int64_t>(blockIdx.y) * kRowsPerBlock;
  const int64_t row0 = rowblk + wave * kRowsPerWave;
  const bool active = col0 < cols && row0 < rows;   // cols and rows are multiples of 32: whole patches only

  uint4 raw[32];
  if (active) {
#pragma unroll
    for (int r = 0; r < 32; ++r) raw[r] = *reinterpret_cast<const uint4*>(x + (row0 + r) * ld + col0);
  } else {
#pragma unroll
    for (int r = 0; r < 32; ++r) raw[r] = make_uint4(0u, 0u, 0u, 0u);
  }

  if (kRow) {
#pragma unroll   // fully: a partly unrolled loop indexes raw[] at run time, which puts the whole patch in scratch memory
    for (int r = 0; r < 32; ++r) {
      float v[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) v[c] = elem(raw[r], c);
      float m = 0.0f;
#pragma unroll
      for (int c = 0; c < 8; ++c) m = fmaxf(m, fabsf(v[c]));
      m = fmaxf(m, lane_xor1(m));   // a 32-column block is four neighbouring lanes
      m = fmaxf(m, lane_xor2(m));
      float inv;
      const uint32_t sc = ue8m0_scale(m, inv);
#pragma unroll
      for (int c = 0; c < 8; ++c) v[c] *= inv;
      uint32_t dr[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if (kSR) draws8(static_cast<uint32_t>(col0 >> 3), static_cast<uint32_t>(row0 + r), 0u, key0, key1, dr);
      const uint32_t codes = encode8<kSR>(v, dr);
      if (active) {
        *reinterpret_cast<uint32_t*>(row_codes + (row0 + r) * (cols / 2) + col0 / 2) = codes;
        if ((lane & 3) == 0) st_row_scales[(wave * kRowsPerWave + r) * 16 + (lane >> 2)] = static_cast<uint8_t>(sc);
      }
      // keep the scheduler from interleaving all 32 rows' temporaries on top of the 128 registers of the patch
      if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
    }
  }

  if (kRow && kCol) {
    // Opaque to the optimiser (no instruction emitted): otherwise it recognises the row pass's unpacked values
    // in the column pass and keeps all 256 of them alive on top of the 128 registers of the patch.
#pragma unroll
    for (int r = 0; r < 32; ++r) asm volatile("" : "+v"(raw[r].x), "+v"(raw[r].y), "+v"(raw[r].z), "+v"(raw[r].w));
  }
  if (kCol) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      float w[32];
#pragma unroll
      for (int r = 0; r < 32; ++r) w[r] = elem(raw[r], c);
      if (kRht) rht32(w, sign_mask);
      float m = 0.0f;
#pragma unroll
      for (int r = 0; r < 32; ++r) m = fmaxf(m, fabsf(w[r]));
      float inv;
      const uint32_t sc = ue8m0_scale(m, inv);
      uint32_t out[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float v[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = w[8 * g + t] * inv;
        uint32_t dr[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (kSR) draws8(static_cast<uint32_t>((row0 >> 3) + g), static_cast<uint32_t>(col0 + c), 1u, key0, key1, dr);
        out[g] = encode8<kSR>(v, dr);
      }
      *reinterpret_cast<uint4*>(st_col_codes + ((c * 4 + wave) * kSlot + lane) * 16) = make_uint4(out[0], out[1], out[2], out[3]);
      st_col_scales[(c * 4 + wave) * 64 + lane] = static_cast<uint8_t>(sc);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  __syncthreads();

  const int tile_cols = static_cast<int>(cols - colblk < kWaveCols ? cols - colblk : kWaveCols);
  const int tile_groups = static_cast<int>((rows - rowblk < kRowsPerBlock ? rows - rowblk : kRowsPerBlock) / 32);   // 32-row groups in this tile
  if (kRow) {
    // 128 rows x (tile_cols / 32) scale bytes; a full tile row is 16 contiguous bytes
    const int r = tid & 127, half = tid >> 7;   // two threads per row, 8 bytes each
    const int64_t row = rowblk + r;
    if (row < rows) {
      const uint8_t* src = st_row_scales + r * 16 + half * 8;
      uint8_t* dst = row_scales + row * (cols / 32) + colblk / 32 + half * 8;
      const int nb = tile_cols / 32 - half * 8;
      if (nb >= 8 && ((cols / 32) & 7) == 0) {
        *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(src);
      } else {
        for (int b = 0; b < nb && b < 8; ++b) dst[b] = src[b];
      }
    }
  }
  if (kCol) {
    const int64_t code_ld = rows / 2, scale_ld = rows / 32;
    const bool wide = (code_ld & 15) == 0;
#pragma unroll 1
    for (int i = 0; i < 8; ++i) {
      const int q = i * kThreads + tid;   // 2048 pieces of 16 bytes: column j, 32-row group g
      const int j = q >> 2, g = q & 3;
      if (j >= tile_cols || g >= tile_groups) continue;
      const int lj = j >> 3, c = j & 7;
      const uint4 v = *reinterpret_cast<const uint4*>(st_col_codes + ((c * 4 + g) * kSlot + lj) * 16);
      uint8_t* dst = col_codes + (colblk + j) * code_ld + (rowblk + 32 * g) / 2;
      if (wide) {
        *reinterpret_cast<uint4*>(dst) = v;
      } else {
        reinterpret_cast<uint32_t*>(dst)[0] = v.x;
        reinterpret_cast<uint32_t*>(dst)[1] = v.y;
        reinterpret_cast<uint32_t*>(dst)[2] = v.z;
        reinterpret_cast<uint32_t*>(dst)[3] = v.w;
      }
    }
#pragma unroll 1
    for (int i = 0; i < 2; ++i) {
      const int j = i * kThreads + tid;   // one column: up to 4 scale bytes
      if (j >= tile_cols) continue;
      const int lj = j >> 3, c = j & 7;
      uint8_t* dst = col_scales + (colblk + j) * scale_ld + rowblk / 32;
      for (int g = 0; g < tile_groups; ++g) dst[g] = st_col_scales[(c * 4 + g) * 64 + lj];
    }
  }
}

template <bool kRow, bool kCol, bool kRht>
void dispatch(const QuantizeArgs& a, dim3 grid, hipStream_t s) {
  const uint16_t* x = static_cast<const uint16_t*>(a.x);
  if (a.sr)
    hipLaunchKernelGGL((quantize_mx_kernel<kRow, kCol, kRht, true>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld,
                       a.sign_mask, a.key0, a.key1, a.row_codes, a.row_scales, a.col_codes, a.col_scales);
  else
    hipLaunchKernelGGL((quantize_mx_kernel<kRow, kCol, kRht, false>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld,
                       a.sign_mask, a.key0, a.key1, a.row_codes, a.row_scales, a.col_codes, a.col_scales);
}

__global__ void mx_tensor_scale_kernel(float* row_ts, float* col_ts) {
  // MXFP4 has no tensor-level scale: s_dec = 1; the amax slot is not computed.
  if (row_ts) { row_ts[0] = 1.0f; row_ts[1] = 0.0f; }
  if (col_ts) { col_ts[0] = 1.0f; col_ts[1] = 0.0f; }
}

}  // namespace

hipError_t launch_quantize_mx(const QuantizeArgs& a, hipStream_t s) {
  const dim3 grid(static_cast<unsigned>((a.cols + kWaveCols - 1) / kWaveCols),
                  static_cast<unsigned>((a.rows + kRowsPerBlock - 1) / kRowsPerBlock));
  hipLaunchKernelGGL(mx_tensor_scale_kernel, dim3(1), dim3(1), 0, s, a.want_row ? a.row_ts : nullptr,
                     a.want_col ? a.col_ts : nullptr);
  if (a.want_row && a.want_col) {
    if (a.rht) dispatch<true, true, true>(a, grid, s); else dispatch<true, true, false>(a, grid, s);
  } else if (a.want_row) {
    dispatch<true, false, false>(a, grid, s);
  } else {
    if (a.rht) dispatch<false, true, true>(a, grid, s); else dispatch<false, true, false>(a, grid, s);
  }
  return hipGetLastError();
}

}  // namespace nvfp4
