// Measurement aids of bench.py for gfx950 -- not part of the NVFP4 library and not a step of the method.
//
//   bench_mfma_rate     a register-only loop of the FP16 matrix instruction the two-pass NVFP4 GEMM runs on
//                       (v_mfma_f32_16x16x32_f16): no memory or LDS traffic, 16 independent accumulators per
//                       wavefront, so timing it gives the rate the matrix pipe sustains on this board under its
//                       power limit for operand values of a given kind.  bench.py quotes it beside the published
//                       peak ("matrix_pipe_context").
//   bench_mfma_rate_gemm_block  the same with the GEMM kernel's own register block: one workgroup of 4 wavefronts
//                       per CU (one per SIMD), 8 x 8 accumulators from 8 + 8 operand registers, so that an operand
//                       register serves 8 instructions in a row as it does there (which costs less power: this loop
//                       runs about a fifth faster than the 4 x 4 one on the same values).
//   bench_stream_copy   a plain device copy of known size (16 bytes per lane and trip, grid-stride): under
//                       rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings calibrate the counters against known
//                       HBM traffic, and its time is the box's plain streaming bandwidth.
//
// Built by __graft_entry__.build() into libbench_probe.so beside bench.py.  Plain C ABI: device pointers, sizes, a
// hipStream_t as void*; returns 0 or -1 (bad argument) / -5 (launch error).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));
typedef float probe_float4 __attribute__((ext_vector_type(4)));

constexpr int kProbeWorkgroups = 512;   // two workgroups of 4 wavefronts per CU

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
  return x;
}

// one FP16 operand value of kind 0 (constant 1), 1 (uniform in [-2, 2) with all mantissa bits in use) or
// 2 (an E2M1 value times an E4M3 block scale, the values the NVFP4 GEMM multiplies)
__device__ __forceinline__ _Float16 probe_value(int kind, uint32_t h) {
  if (kind == 0) return static_cast<_Float16>(1.0f);
  if (kind == 1) return static_cast<_Float16>((static_cast<float>(h >> 8) - 8388608.0f) * (1.0f / 4194304.0f));
  const float grid[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
  const float v = grid[h & 7];
  const float sc = __builtin_amdgcn_cvt_f32_fp8(static_cast<int>(40 + ((h >> 4) & 31)), 0);   // E4M3 scales 2^-2 .. 2^1.9
  return static_cast<_Float16>(((h >> 3) & 1) ? -v * sc : v * sc);
}

__global__ __launch_bounds__(256) void mfma_rate_kernel(int kind, long long iters, float* __restrict__ out) {
  const uint32_t tid = blockIdx.x * 256 + threadIdx.x;
  probe_half8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      a[i][e] = probe_value(kind, probe_hash(tid * 64 + i * 8 + e));
      b[i][e] = probe_value(kind, probe_hash(tid * 64 + 32 + i * 8 + e));
    }
  probe_float4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = probe_float4{0.0f, 0.0f, 0.0f, 0.0f};
  for (long long it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  probe_float4 t = probe_float4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) t += acc[i][j];
  out[tid] = t[0] + t[1] + t[2] + t[3];
}

__global__ __launch_bounds__(256) void mfma_rate_gemm_block_kernel(int kind, long long iters, float* __restrict__ out) {
  const uint32_t tid = blockIdx.x * 256 + threadIdx.x;
  probe_half8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      a[i][e] = probe_value(kind, probe_hash(tid * 128 + i * 8 + e));
      b[i][e] = probe_value(kind, probe_hash(tid * 128 + 64 + i * 8 + e));
    }
  probe_float4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = probe_float4{0.0f, 0.0f, 0.0f, 0.0f};
  for (long long it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  probe_float4 t = probe_float4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) t += acc[i][j];
  out[tid] = t[0] + t[1] + t[2] + t[3];
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = static_cast<size_t>(gridDim.x) * 256;
  for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

extern "C" {

int bench_mfma_probe_threads(void) { return kProbeWorkgroups * 256; }

// operand_kind 0 ones, 1 random FP16, 2 NVFP4-like values; iters 1 .. 2^24 loop trips of 16 MFMAs per wavefront;
// out: device, float[bench_mfma_probe_threads()], one checksum per thread; flops: host, the launch's flop count.
int bench_mfma_rate(int operand_kind, int64_t iters, float* out, double* flops, void* stream) {
  if (!out || !flops || reinterpret_cast<uintptr_t>(out) % 4) return -1;
  if (operand_kind < 0 || operand_kind > 2 || iters <= 0 || iters > (int64_t{1} << 24)) return -1;
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(kProbeWorkgroups), dim3(256), 0, static_cast<hipStream_t>(stream), operand_kind,
                     static_cast<long long>(iters), out);
  *flops = static_cast<double>(kProbeWorkgroups) * 4.0 * static_cast<double>(iters) * 16.0 * (2.0 * 16 * 16 * 32);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

// The same with 256 workgroups and 64 MFMAs per trip (8 x 8 accumulators); iters 1 .. 2^22; out as above (the first
// half of it is written).
int bench_mfma_rate_gemm_block(int operand_kind, int64_t iters, float* out, double* flops, void* stream) {
  if (!out || !flops || reinterpret_cast<uintptr_t>(out) % 4) return -1;
  if (operand_kind < 0 || operand_kind > 2 || iters <= 0 || iters > (int64_t{1} << 22)) return -1;
  hipLaunchKernelGGL(mfma_rate_gemm_block_kernel, dim3(kProbeWorkgroups / 2), dim3(256), 0, static_cast<hipStream_t>(stream),
                     operand_kind, static_cast<long long>(iters), out);
  *flops = static_cast<double>(kProbeWorkgroups / 2) * 4.0 * static_cast<double>(iters) * 64.0 * (2.0 * 16 * 16 * 32);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

// dst[0 .. bytes) = src[0 .. bytes); both device, 16-byte aligned, bytes a multiple of 16.
int bench_stream_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || bytes == 0 || bytes % 16 || reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(dst) % 16)
    return -1;
  hipLaunchKernelGGL(stream_copy_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

}  // extern "C"
