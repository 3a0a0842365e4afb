// Host-side launch interfaces between the C ABI (api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace nvfp4 {

// Kernels that need more dynamic LDS than the default limit have it raised once per device (the attribute belongs to
// the kernel on the current device).  One flag bit per device ordinal; setting the attribute again is harmless, so
// two host threads racing through here at worst both set it.
struct PerDeviceOnce {
  std::atomic<uint64_t> done{0};
};
inline hipError_t ensure_dynamic_lds(const void* kernel, int bytes, PerDeviceOnce& once) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = uint64_t{1} << (dev & 63);
  if (dev < 64 && (once.done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && dev < 64) once.done.fetch_or(bit, std::memory_order_release);
  return e;
}

struct QuantizeArgs {
  const void* x;
  int64_t rows, cols, ld;
  bool want_row, want_col, rht, sr, block2d;
  bool row_rht = false;    // the row copy is rotated too (16-point, along the columns); sign_mask then holds the 16 signs
  bool scale_per_row = false;   // one tensor-level scale per row of each copy (App. B.1, last sentence); row_ts / col_ts
                                // then hold 2 * outer floats, ws the words of quantize_rowscale_workspace_words
  int rht_dim;             // 0, or the rotation size: 2, 4, 16, 32, 128 (NVFP4); 32 (MXFP4)
  uint32_t sign_mask;      // the sign diagonal: d <= 16: its d bits repeated over the low 16 bits; 32: its 32 bits
  uint32_t sign_words[4];  // the sign diagonal's bits, first rht_dim of the 128 meaningful
  uint32_t key0, key1;
  uint32_t* ws;  // device workspace: [0] raw amax bits, [1] rotated amax bits, [2] amax bits of the row-rotated
                 // tensor (row_rht only), then per-workgroup partials
  // The two passes can run apart: without do_amax, ws is any two device words holding the amax bits (raw, rotated);
  // without do_cast only the amax is computed, and amax_copy (if set) receives the two words as well.
  bool do_amax = true, do_cast = true;
  uint32_t* amax_copy = nullptr;
  uint8_t *row_codes, *row_scales;
  float* row_ts;
  uint8_t *col_codes, *col_scales;
  float* col_ts;
};
hipError_t launch_quantize(const QuantizeArgs& a, hipStream_t s);
// NVFP4 with a 32- or 128-point rotation of the col copy (rotation groups span several 16-row groups)
hipError_t launch_quantize_wide(const QuantizeArgs& a, hipStream_t s);
// NVFP4 with the row copy rotated as well (row_rht; the col copy absent, plain or rotated with d = 16)
hipError_t launch_quantize_rowrot(const QuantizeArgs& a, hipStream_t s);
// MXFP4 mode (1x32 blocks, UE8M0 scales, one pass, no workspace); sign_mask holds 32 bits
hipError_t launch_quantize_mx(const QuantizeArgs& a, hipStream_t s);
// NVFP4 with one tensor-level scale per row of each copy (1x16 blocks, col copy plain or rotated with d = 16)
hipError_t launch_quantize_rowscale(const QuantizeArgs& a, hipStream_t s);
size_t quantize_rowscale_workspace_words(int64_t rows, int64_t cols);
size_t quantize_workspace_bytes(int64_t rows, int64_t cols);

// One K-contiguous operand: codes [outer, K/2], scales [outer, K/16], ts = {s_dec, amax}.
struct Operand {
  const uint8_t* codes;
  const uint8_t* scales;
  const float* ts;
  int64_t outer;
  int ts_per_row = 0;   // 0: ts = {s_dec, amax}; 1: ts = s_dec of every row, then the amax of every row (App. B.1, last sentence)
  const void* fp16 = nullptr;   // the copy already decoded to FP16 [outer, K] (nvfp4_predecode), or null
};
struct GemmArgs {
  Operand a, b;  // D[m, n] = sum_k A[m, k] B[n, k]
  int64_t K;
  void* d;
  int64_t ldd;
  bool out_bf16;
  bool accumulate;   // FP32 output only: D <- D + result
  bool mx = false;   // operands are MXFP4 (UE8M0 scale per 32) instead of NVFP4
  void* workspace;        // optional: room for both operands decoded to FP16
  size_t workspace_bytes;
};
hipError_t launch_gemm(const GemmArgs& g, hipStream_t s);
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
bool gemm_two_pass_usable(const GemmArgs& g);
hipError_t launch_gemm_two_pass(const GemmArgs& g, hipStream_t s);
// Decodes one operand (codes [outer, K/2], scales [outer, K/16]) to FP16 [outer, K]
hipError_t launch_predecode(const Operand& op, int64_t K, void* fp16_out, hipStream_t s);

struct DequantArgs {
  Operand q;
  int64_t K;
  bool undo_rht;
  int rht_dim;             // size of the rotation to undo
  uint32_t sign_mask;      // as in QuantizeArgs
  uint32_t sign_words[4];
  void* out;
  int64_t ld_out;
  bool out_bf16;
};
hipError_t launch_dequantize(const DequantArgs& d, hipStream_t s);
hipError_t launch_dequantize_mx(const DequantArgs& d, hipStream_t s);   // scales are UE8M0 per 32

hipError_t run_selftest(uint64_t* mismatches_dev, hipStream_t s);

// Host Philox4x32-10, used only to derive the sign diagonal from a seed (16 bits, or 32 for the MXFP4 mode).
uint32_t host_rht_sign_mask(uint64_t seed);
uint32_t host_rht_sign_mask32(uint64_t seed);
void host_rht_sign_words(uint64_t seed, uint32_t words[4]);   // all 128 bits of the same Philox call

// MXFP4 GEMM on the scaled FP4 MFMA (scales per 32 are UE8M0); K must be a multiple of 128.
hipError_t launch_gemm_mx(const GemmArgs& g, hipStream_t s);

}  // namespace nvfp4
