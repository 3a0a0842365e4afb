/*
 * nvfp4.h -- C ABI of the MI355X (gfx950) NVFP4 quantize-and-GEMM library.
 *
 * Implements the per-linear-layer hot path of "Pretraining Large Language
 * Models with NVFP4" (arXiv 2509.25149): two-level scaled E2M1 quantization
 * (Sec. 2, App. B), 16x16 weight blocks (Sec. 4.3), the 16-point random
 * Hadamard rotation of the Wgrad operands (Sec. 4.2, App. C), stochastic
 * rounding of gradients (Sec. 4.4) and the block-scaled GEMM with FP32
 * accumulation (Sec. 2, App. B.3 Eq. 5).
 *
 * General rules
 *   - Every data pointer is a DEVICE pointer unless marked "host".  The
 *     library never allocates, frees or retains device memory: the caller
 *     owns every buffer, including the small workspace.
 *   - Every call only enqueues kernels on the given HIP stream (a
 *     hipStream_t passed as void*; NULL is the default stream) and returns
 *     without waiting.  Argument checks are synchronous: a call that returns
 *     an error has enqueued nothing.
 *   - Return value: NVFP4_OK (0) or a negative nvfp4_status.
 *   - Data-dependent trouble never aborts: a tensor containing Inf/NaN yields
 *     amax = Inf/NaN in tensor_scale[1] of every copy written (rotated or not;
 *     NVFP4 formats) and unspecified codes.
 *   - Calls on different streams with disjoint buffers are independent, from
 *     any host thread.  The only state the library keeps is a per-device note
 *     that a kernel's shared-memory limit has been raised (set on the first
 *     launch of that kernel on the device; idempotent).
 *
 * Storage format (the paper fixes the number formats, not the layout)
 *   - E2M1 code: bit 3 sign, bits 2..0 index into {0, .5, 1, 1.5, 2, 3, 4, 6}
 *     (Sec. 2).  Two codes per byte, element 2j in the low nibble.
 *   - Block scale: one E4M3 byte (bias 7, max 448, App. B.1) per 16
 *     consecutive elements along the copy's contiguous dimension.
 *   - "row copy" of a logical [rows, cols] tensor: codes [rows, cols/2] bytes,
 *     scales [rows, cols/16] bytes, blocks along cols.
 *   - "col copy": the row-wise quantization of the transposed tensor, stored
 *     transposed: codes [cols, rows/2] bytes, scales [cols, rows/16] bytes,
 *     blocks along rows.  This is the operand layout a GEMM contracting over
 *     `rows` needs (Sec. 4.3: scaling runs along the dot-product dimension).
 *   - tensor_scale: float[2] per copy, [0] = s_dec = 1/s_enc (App. B.1 Eq. 1),
 *     [1] = the amax it was derived from (in the rotated space for a rotated
 *     copy, App. C).
 *   - With 16x16 blocks (weights) one scale per tile is replicated into every
 *     1x16 slot of both copies, so the col copy is the exact transpose of the
 *     row copy (Sec. 4.3).
 */
#ifndef NVFP4_H_
#define NVFP4_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void* nvfp4_stream_t; /* a hipStream_t */

typedef enum nvfp4_status {
  NVFP4_OK = 0,
  NVFP4_ERR_INVALID_ARG = -1,  /* null pointer, unknown enum value */
  NVFP4_ERR_BAD_SHAPE = -2,    /* rows or cols not a positive multiple of 16, ld too small */
  NVFP4_ERR_MISSING_COPY = -3, /* the copy an operation needs is absent from the descriptor */
  NVFP4_ERR_MISMATCH = -4,     /* operands disagree on K, rotation size or rotation seed */
  NVFP4_ERR_HIP = -5,          /* a HIP runtime call failed (launch error) */
  NVFP4_ERR_WORKSPACE = -6     /* workspace missing or too small */
} nvfp4_status;

enum { NVFP4_LAYOUT_ROW = 1, NVFP4_LAYOUT_COL = 2 };       /* layout mask bits */
/* Extra layout mask bit of nvfp4_quantize: rotate the row copy too.  Sec. 4.2 restricts the random Hadamard
 * transform to the Wgrad operands (the col copies); App. E.4.1 ablates it on the operands of Fprop and Dgrad, whose
 * contraction runs along the row copy's columns.  With this bit every aligned group of 16 consecutive columns of a
 * row is multiplied by the sign diagonal of rht_seed and by H_16 before scaling (App. C; same stage order and
 * normalisation as for the col copy), and the row copy's tensor scale comes from the amax of the values rotated
 * that way.  NVFP4 with 1x16 blocks only, NVFP4_LAYOUT_ROW required, the col copy (if asked for) plain or rotated
 * with d = 16; not accepted by nvfp4_quantize_with_amax.  The descriptor records it as row_has_rht = 16. */
enum { NVFP4_LAYOUT_ROW_RHT = 4 };
/* Extra layout mask bit of nvfp4_quantize: a tensor-level scale of finer granularity.  App. B.1 (last sentence) notes
 * that the global scale may span a row or a block instead of the whole tensor, which saves the extra pass over device
 * memory that the tensor's amax costs.  With this bit Eq. 1 is evaluated once per row of each emitted copy's
 * K-contiguous storage, with that row's amax: per logical row for the row copy, per logical column (over the rotated
 * values, App. C) for the col copy -- the one granularity that stays constant along the contraction, so that
 * nvfp4_gemm can still apply the two tensor-level factors after the sum (Eq. 5): D[m, n] gets s_dec^A[m] * s_dec^B[n].
 * Eq. 2-4 are unchanged.  tensor_scale of a copy then is float[2 * outer] (outer = rows for the row copy, cols for
 * the col copy): s_dec of every row, then the amax of every row.  A row copy asked for alone (up to 32768 columns) is
 * produced in ONE pass over the tensor -- a workgroup holds its row in registers; a col copy's amax spans all rows of
 * the tensor, so calls that emit it still read the tensor twice.  NVFP4 with 1x16 blocks only (a 16x16 weight tile's
 * scale has to serve both orientations, Sec. 4.3), rht_on_col 0, 1 or 16, not with NVFP4_LAYOUT_ROW_RHT, not accepted
 * by nvfp4_quantize_with_amax.  Operands of either granularity mix freely in nvfp4_gemm (per-row activations with a
 * per-tensor 16x16 weight).  Non-finite input is reported in the amax of the rows (row copy) it occurs in; the col
 * copy's rotated maxima skip NaNs.  The descriptor records it as scale_per_row = 1. */
enum { NVFP4_LAYOUT_ROW_SCALES = 8 };
/* block_dim.  NVFP4_BLOCK_MX32 selects the paper's comparison format MXFP4 instead of NVFP4 (Sec. 2, App. B.4,
 * Sec. 5): blocks of 32 along the copy's contiguous dimension, one UE8M0 byte per block (2^(byte - 127), amax_b / 6
 * rounded up to a power of two), no tensor-level scale (tensor_scale = {1, 0}), scales [.., ../32] bytes, a 32-point
 * rotation (all 32 bits of the sign word) when rht_on_col is set, rows and cols multiples of 32, no workspace.  The
 * col copy draws its own random numbers: element (i, j) uses counter (i / 8, j, 1, 0), word (i % 8) / 2.
 * nvfp4_gemm on two MXFP4 tensors runs on the chip's block-scaled FP4 matrix instruction (K a multiple of 128). */
enum { NVFP4_BLOCK_1x16 = 1, NVFP4_BLOCK_16x16 = 16, NVFP4_BLOCK_MX32 = 32 };
enum { NVFP4_ROUND_RNE = 0, NVFP4_ROUND_SR = 1 };          /* rounding */
enum { NVFP4_OP_FPROP = 0, NVFP4_OP_DGRAD = 1, NVFP4_OP_WGRAD = 2 };
/* NVFP4_OUT_F32_ACCUMULATE (nvfp4_gemm only): D <- D + result in FP32, for weight gradients that are
 * accumulated over micro-batches in FP32 (Sec. 4.1, last paragraph). */
enum { NVFP4_OUT_F32 = 0, NVFP4_OUT_BF16 = 1, NVFP4_OUT_F32_ACCUMULATE = 2 };
enum { NVFP4_COPY_ROW = 0, NVFP4_COPY_COL = 1 };

/*
 * Descriptor of a quantized tensor.  Caller-owned plain struct; the caller
 * fills the pointers of the copies it wants before nvfp4_quantize, which
 * fills the remaining fields.  Unused copies have NULL pointers.
 */
typedef struct nvfp4_qtensor {
  int64_t rows, cols;       /* logical shape of the source tensor */
  void* row_codes;          /* [rows, cols/2] bytes */
  void* row_scales;         /* [rows, cols/16] bytes */
  float* row_tensor_scale;  /* float[2]: s_dec, amax */
  void* col_codes;          /* [cols, rows/2] bytes */
  void* col_scales;         /* [cols, rows/16] bytes */
  float* col_tensor_scale;  /* float[2]: s_dec, amax */
  int32_t layout_mask;      /* which copies hold data (set by nvfp4_quantize) */
  int32_t block_dim;        /* NVFP4_BLOCK_* used */
  int32_t rounding;         /* NVFP4_ROUND_* used */
  int32_t col_has_rht;      /* 0, or the size d of the rotation applied to the col copy */
  uint64_t rht_seed;        /* seed of the sign diagonal, if rotated */
  int32_t row_has_rht;      /* 0, or 16: the row copy is rotated along its columns (NVFP4_LAYOUT_ROW_RHT) */
  int32_t scale_per_row;    /* 0: tensor_scale is float[2]; 1: float[2 * outer] per copy (NVFP4_LAYOUT_ROW_SCALES) */
  void* row_fp16;           /* NULL, or the row copy decoded to FP16 by nvfp4_predecode (rows x cols elements) */
  void* col_fp16;           /* NULL, or the col copy decoded to FP16 by nvfp4_predecode (cols x rows elements) */
} nvfp4_qtensor;

/*
 * Byte counts for one copy of a [rows, cols] tensor and for the workspace
 * nvfp4_quantize needs (host pointers, any may be NULL).  codes_bytes and
 * scales_bytes are the same for the row and the col copy.
 */
int nvfp4_quantized_sizes(int64_t rows, int64_t cols, size_t* codes_bytes, size_t* scales_bytes,
                          size_t* workspace_bytes);

/*
 * Quantize a bf16 tensor to NVFP4 (App. B Eq. 1-4).
 *   x            device, bf16 [rows, cols], row-major with leading dimension ld (elements)
 *   layout_mask  NVFP4_LAYOUT_ROW | NVFP4_LAYOUT_COL: which copies to emit
 *                (| NVFP4_LAYOUT_ROW_RHT: the row copy rotated as well;
 *                 | NVFP4_LAYOUT_ROW_SCALES: one tensor-level scale per row of each copy)
 *   block_dim    1x16 (activations, gradients) or 16x16 (weights, Sec. 4.3)
 *   rounding     RNE (weights, activations) or SR (gradients), Sec. 4.4
 *   rht_on_col   rotate the col copy: every aligned group of d consecutive
 *                rows of a column is multiplied by the sign diagonal and the
 *                d-point Hadamard matrix before scaling (Sec. 4.2, App. C).
 *                0 = no rotation; 1 = the format's own size (d = 16, the
 *                paper's choice; 32 for MXFP4); 2, 4, 16, 32 or 128 = that
 *                size (the other sizes of the ablation in Sec. 4.2 "Hadamard
 *                matrix size" and App. E.4; NVFP4 only).  rows must be a
 *                multiple of d.  Not allowed with 16x16 blocks.  Butterfly
 *                stages h = 1, 2, .., d/2 in this order, then one multiply
 *                by the binary32 nearest to 1/sqrt(d).
 *   rht_seed     selects the sign diagonal: sign i is bit i of the 128 bits of
 *                one Philox call (nvfp4_rht_sign_mask gives the first 16)
 *   sr_seed      key of the Philox4x32-10 stream used for SR; element (i, j)
 *                uses counter (j/8, i, 0, 0), 16 bits per element, so both
 *                copies round with the same draw
 *   out          host pointer to the descriptor; its copy pointers for the
 *                requested layouts must be set (device memory sized by
 *                nvfp4_quantized_sizes)
 *   workspace    device, >= workspace_bytes; contents irrelevant on entry
 * The global amax costs a first pass over x (App. B.1); the second pass
 * scales, rounds, packs and writes every requested copy.
 */
int nvfp4_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, int layout_mask,
                   int block_dim, int rounding, int rht_on_col, uint64_t rht_seed, uint64_t sr_seed,
                   nvfp4_qtensor* out, void* workspace, size_t workspace_bytes,
                   nvfp4_stream_t stream);

/*
 * nvfp4_quantize for callers that cannot allocate device memory or carry a workspace around: code running under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical results as nvfp4_quantize, minus the workspace: the amax pass's scratch lives in a fixed device
 * array of NVFP4_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process ends).
 * The call allocates and frees nothing.  Tensors whose workspace need (nvfp4_quantized_sizes) exceeds
 * NVFP4_STATIC_SCRATCH_BYTES are refused with NVFP4_ERR_WORKSPACE (enough for 87376 workgroup tiles of 128 rows x 512
 * columns, e.g. 65536 x 81920 elements); MXFP4 needs no scratch and has no limit.  Nothing in the array has to start
 * at zero (every word is written before it is read), and it keeps the last call's contents.  All calls on one GPU
 * share the array: two calls that overlap in time on one GPU (different streams, or different host threads) race;
 * calls on one stream, or ordered by events, are fine.  The first call on a device looks the array's address up
 * (hipGetSymbolAddress) and must not be made under stream capture; later calls may be.
 */
enum { NVFP4_STATIC_SCRATCH_BYTES = 1 << 20 };
int nvfp4_quantize_static(const void* x, int64_t rows, int64_t cols, int64_t ld, int layout_mask, int block_dim,
                          int rounding, int rht_on_col, uint64_t rht_seed, uint64_t sr_seed, nvfp4_qtensor* out,
                          nvfp4_stream_t stream);

/*
 * The two passes of nvfp4_quantize as separate calls.  App. B.1 counts the global amax as an extra pass through
 * device memory; a caller that knows the amax beforehand (a weight whose amax the optimizer step tracked, an amax
 * kept from the previous iteration) or has to combine it over the shards of a larger tensor (a max all-reduce
 * between the two calls) runs only what it needs.  NVFP4 only (MXFP4 has no tensor-level scale).
 *
 * nvfp4_amax: pass 1.  amax_out is device memory, float[2]: { max |x|, max |rotated x| } (the second is 0 without
 * rht_on_col, or non-finite like the first for a tensor holding Inf/NaN; it is what Eq. 1 uses for a rotated col copy, App. C).  rht_on_col, rht_seed, workspace as in
 * nvfp4_quantize (same workspace size).
 *
 * nvfp4_quantize_with_amax: pass 2.  amax_in is device memory, float[2] laid out as nvfp4_amax writes it, read by the
 * kernels when they run; values must be >= 0 and finite.  Every other argument as in nvfp4_quantize; no workspace.
 * With amax_in = this tensor's own amax the result is bit-identical to nvfp4_quantize's.  A larger amax only moves
 * the block scales along the E4M3 grid; with a smaller one block scales saturate at 448 and codes at +-6
 * (Eq. 3-4).  tensor_scale[1] reports the amax that was used.
 */
int nvfp4_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int rht_on_col, uint64_t rht_seed,
               float* amax_out, void* workspace, size_t workspace_bytes, nvfp4_stream_t stream);
int nvfp4_quantize_with_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int layout_mask, int block_dim,
                             int rounding, int rht_on_col, uint64_t rht_seed, uint64_t sr_seed,
                             const float* amax_in, nvfp4_qtensor* out, nvfp4_stream_t stream);

/*
 * Block-scaled GEMM (Eq. 5): D[m, n] = s_dec^A s_dec^B sum_b sA[m,b] sB[n,b]
 * sum_{k in b} A[m,k] B[n,k], FP32 accumulation (s_dec^A[m] s_dec^B[n] for operands
 * quantized with NVFP4_LAYOUT_ROW_SCALES).  `op` picks the copies:
 *   FPROP  Y  = X W      A = row copy of X [M,K],   B = col copy of W [K,N] (-> [N,K])
 *   DGRAD  dX = dY W^T   A = row copy of dY [M,K],  B = row copy of W [N,K]
 *   WGRAD  dW = A^T B    A = col copy of the first tensor [K,M] (-> [M,K]),
 *                        B = col copy of the second [K,N] (-> [N,K])
 * For every op the two copies it reads must agree on rotation size and seed
 * (col_has_rht / row_has_rht of the copy read; App. C: the two rotations cancel
 * in the product only if they are the same), else NVFP4_ERR_MISMATCH.
 * D is device memory, 16-byte aligned, [M, N] row-major with leading dimension
 * ldd -- a multiple of 4 elements for FP32 and of 8 for bf16 (results leave in
 * 16-byte pieces), else NVFP4_ERR_BAD_SHAPE -- FP32 or bf16 (bf16 =
 * round-to-nearest-even of the FP32 result).  With
 * NVFP4_OUT_F32_ACCUMULATE, D is FP32 and is read: every element becomes
 * fp32(D_old + result), one FP32 addition after the FP32 result is formed.
 * workspace: optional device scratch, 256-byte aligned.  With at least
 * nvfp4_gemm_workspace_bytes(M, N, K) bytes (and K a multiple of 64) the call
 * first decodes both operands to FP16 (value * block scale, exact) into it and
 * then runs an FP16 MFMA GEMM with no decode work in its loop; with NULL or
 * too little room it runs a fused kernel that decodes inside the GEMM loop
 * (slower, no scratch).  Both give the same result up to FP32 summation order.
 * (With both operands decoded beforehand by nvfp4_predecode and no split last
 * round of tiles the FP16 GEMM needs nothing of the workspace and runs without.)
 * The workspace contents are scratch: undefined afterwards, free for reuse once
 * the call's kernels have run.
 */
int nvfp4_gemm(const nvfp4_qtensor* a, const nvfp4_qtensor* b, int op, void* d, int out_dtype,
               int64_t ldd, void* workspace, size_t workspace_bytes, nvfp4_stream_t stream);

/*
 * Decode one copy of an NVFP4 tensor to FP16 once (value * block scale, exact), for the nvfp4_gemm calls that follow.
 * A weight is quantized once per optimizer step and then serves Fprop and Dgrad of every micro-batch (Sec. 4.3: the
 * same quantized weight in both passes; Sec. 4.1: gradients accumulate over micro-batches): without this every
 * nvfp4_gemm call on its two-pass route decodes the operand again.
 *   q           host descriptor of a quantized NVFP4 tensor (not MXFP4); on success its row_fp16 / col_fp16 field
 *               is set to fp16_out, and nvfp4_gemm reads that instead of decoding (its workspace then only has to
 *               hold the operands still to decode and the partial tiles)
 *   fp16_out    device, 16-byte aligned, outer * K * 2 bytes (outer x K = rows x cols for the row copy, cols x rows for
 *               the col copy; K must be a multiple of 64, NVFP4_ERR_BAD_SHAPE otherwise).  The elements are stored in
 *               the order the GEMM kernel loads them (16 rows x 32 k per KiB), not row by row: the buffer is for
 *               nvfp4_gemm only.  Owned by the caller, must stay valid while the descriptor points to it
 *   fp16_bytes  its size; NVFP4_ERR_WORKSPACE if too small
 * nvfp4_quantize into the same descriptor clears both fields (the codes change), as does any call that rewrites it.
 */
int nvfp4_predecode(nvfp4_qtensor* q, int which_copy, void* fp16_out, size_t fp16_bytes, nvfp4_stream_t stream);

/* Scratch bytes that let nvfp4_gemm take its faster two-pass route (host pointer out):
 * (M + N) * K * 2 for the FP16 operands and up to 64 MiB of FP32 partial tiles when the last
 * round of 256x256 output tiles is partial and gets split along K.
 * Two calls that overlap in time on one GPU need a workspace each. */
int nvfp4_gemm_workspace_bytes(int64_t m, int64_t n, int64_t k, size_t* workspace_bytes);

/*
 * One linear layer, forward and backward, as the sequence of calls above
 * (Sec. 4.1 and its compute-flow figure; Sec. 4.2-4.4 for which operand gets
 * which treatment).  W [d_in, d_out] is quantized by the caller, once per
 * optimizer step, with nvfp4_quantize(ROW | COL, 16x16 blocks) and reused by
 * both calls.  All checks of every step run before anything is enqueued.
 *
 * nvfp4_linear_forward: quantize X [tokens, d_in] (bf16, leading dimension
 *   ldx) with RNE -- row copy for Fprop and, if keep_for_backward, the rotated
 *   col copy Wgrad will need (sign diagonal from rht_seed) -- then
 *   Y [tokens, d_out] = X W (out_dtype FP32 or bf16, leading dimension ldy).
 *   qx: host descriptor with the copy pointers set (nvfp4_quantized_sizes);
 *   it is filled in and must stay alive until nvfp4_linear_backward.
 * nvfp4_linear_backward: quantize dY [tokens, d_out] with stochastic rounding
 *   (key sr_seed), row copy for Dgrad and col copy rotated like qx's, then
 *   dX [tokens, d_in] = dY W^T (dx_dtype FP32 or bf16) and
 *   dW [d_in, d_out] = X^T dY in FP32, added into dw if accumulate_dw
 *   (micro-batch gradient accumulation), stored otherwise.
 *   qdy: host descriptor with both copies' pointers set; scratch for the call.
 * workspace: device, 256-byte aligned, shared by all steps of a call.  At least
 *   the quantizer's need (nvfp4_quantized_sizes) is required; with
 *   nvfp4_linear_workspace_bytes(tokens, d_in, d_out) bytes every GEMM takes
 *   its faster two-pass route.
 */
int nvfp4_linear_workspace_bytes(int64_t tokens, int64_t d_in, int64_t d_out, size_t* workspace_bytes);
int nvfp4_linear_forward(const void* x, int64_t tokens, int64_t d_in, int64_t ldx, const nvfp4_qtensor* qw,
                         int keep_for_backward, uint64_t rht_seed, nvfp4_qtensor* qx, void* y, int out_dtype,
                         int64_t ldy, void* workspace, size_t workspace_bytes, nvfp4_stream_t stream);
int nvfp4_linear_backward(const void* dy, int64_t tokens, int64_t d_out, int64_t lddy, const nvfp4_qtensor* qx,
                          const nvfp4_qtensor* qw, uint64_t sr_seed, nvfp4_qtensor* qdy, void* dx, int dx_dtype,
                          int64_t lddx, float* dw, int64_t lddw, int accumulate_dw, void* workspace,
                          size_t workspace_bytes, nvfp4_stream_t stream);

/*
 * Decode one copy back to FP32 or bf16: value(code) * block scale * s_dec
 * (Sec. 2; App. B.2).  The output has the copy's own orientation: [rows, cols]
 * for the row copy, [cols, rows] for the col copy, leading dimension ld_out.
 * undo_rht rotates each group of d back, d = q->col_has_rht or q->row_has_rht of the chosen copy (NVFP4_ERR_MISMATCH
 * for a copy that is not rotated).
 */
int nvfp4_dequantize(const nvfp4_qtensor* q, int which_copy, int undo_rht, void* out, int out_dtype,
                     int64_t ld_out, nvfp4_stream_t stream);

/* 16-bit sign diagonal for a seed: bit i set means s_i = -1 (App. C). */
uint32_t nvfp4_rht_sign_mask(uint64_t rht_seed);

/*
 * Device self-test of the gfx950 conversion instructions the quantizer relies
 * on, against explicit integer/compare implementations run on the device.
 * mismatches: DEVICE pointer to uint64[5], zeroed by the caller; the kernels
 * add their mismatch counts: [0] FP32->E2M1 RNE over all 2^32 bit patterns,
 * [1] FP32->E2M1 SR over a grid of values x all 2^16 random values (the plain
 * and the accumulating form of the conversion),
 * [2] FP32->E4M3 (and back) over all non-negative finite patterns,
 * [3] the division-free x/6 against IEEE division over the same patterns,
 * [4] FP32->bf16 (the GEMM and dequantize outputs) over all finite patterns.
 * Asynchronous like every other call.
 */
int nvfp4_selftest_conversions(uint64_t* mismatches, nvfp4_stream_t stream);

const char* nvfp4_status_string(int status);
int nvfp4_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NVFP4_H_ */
