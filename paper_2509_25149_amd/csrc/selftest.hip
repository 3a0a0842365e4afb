// On-device check of the gfx950 conversion instructions the quantizer uses
// against explicit compare / integer formulations of the same rounding rules:
// E2M1 round-to-nearest-even with ties to the even code and saturation at 6
// (Sec. 2, Sec. 4 item 4), E2M1 stochastic rounding at 16-bit resolution
// (Sec. 4.4) and E4M3 round-to-nearest-even saturating at 448 (App. B.2).
#include "nvfp4_internal.h"
#include "nvfp4_device.h"

namespace nvfp4 {

namespace {

__device__ __forceinline__ uint32_t ref_e2m1_rne(float v) {
  const float a = fabsf(v);
  uint32_t idx;
  if (a <= 0.25f) idx = 0;
  else if (a < 0.75f) idx = 1;
  else if (a <= 1.25f) idx = 2;
  else if (a < 1.75f) idx = 3;
  else if (a <= 2.5f) idx = 4;
  else if (a < 3.5f) idx = 5;
  else if (a <= 5.0f) idx = 6;
  else idx = 7;
  return ((__float_as_uint(v) >> 31) << 3) | idx;
}

// up iff floor(p * 2^16) + r >= 2^16, p = position between the grid neighbours
__device__ __forceinline__ uint32_t ref_e2m1_sr(float v, uint32_t r16) {
  const float a = fabsf(v);
  const uint32_t s = (__float_as_uint(v) >> 31) << 3;
  if (!(a < 6.0f)) return s | 7u;
  const uint32_t fx = static_cast<uint32_t>(a * 131072.0f);  // exact product, truncation
  uint32_t idx;
  if (a < 2.0f) {
    idx = (fx + r16) >> 16;            // steps of 0.5: 0, .5, 1, 1.5, 2 -> codes 0..4
  } else if (a < 4.0f) {
    idx = (((fx >> 1) + r16) >> 16) + 2;   // steps of 1: 2, 3, 4 -> codes 4, 5, 6
  } else {
    idx = (((fx >> 2) + r16) >> 16) + 4;   // steps of 2: 4, 6 -> codes 6, 7
  }
  return s | idx;
}

__device__ __forceinline__ uint32_t ref_e4m3(float u) {
  if (!(u > 0.0f)) return 0;
  if (u >= 448.0f) return 0x7E;
  if (u < 0.015625f) return static_cast<uint32_t>(rintf(u * 512.0f));
  uint32_t w = __float_as_uint(u);
  w += 0x7FFFFu + ((w >> 20) & 1u);      // RNE on the 20 dropped mantissa bits
  return (w >> 20) - ((127u - 7u) << 3);
}

__global__ __launch_bounds__(256) void selftest_rne_kernel(unsigned long long* bad) {
  unsigned long long local = 0;
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  for (uint64_t w = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; w < (1ull << 32); w += stride) {
    const uint32_t bits = static_cast<uint32_t>(w);
    if ((bits & 0x7FFFFFFFu) > 0x7F800000u) continue;
    const float v = __uint_as_float(bits);
    const uint32_t hw = cvt_rne_pair<0>(0u, v, -v);
    const uint32_t want = ref_e2m1_rne(v) | (ref_e2m1_rne(-v) << 4);
    local += (hw & 0xFFu) != want;
  }
  if (local) atomicAdd(bad, local);
}

__global__ __launch_bounds__(256) void selftest_sr_kernel(unsigned long long* bad) {
  // values: every FP32 pattern whose top 16 bits run over [0, 7.0] and whose low
  // 16 bits take one of 5 patterns; random draws: all 2^16 values.
  const uint32_t low[5] = {0x0000u, 0x0001u, 0x8000u, 0xFFFFu, 0x5555u};
  const uint32_t n_hi = 0x40E1u;
  unsigned long long local = 0;
  const uint32_t vidx = blockIdx.x;  // one value per block
  if (vidx >= n_hi * 5) return;
  const uint32_t bits = ((vidx / 5) << 16) | low[vidx % 5];
  const float v = __uint_as_float(bits);
  for (uint32_t r = threadIdx.x; r < 65536u; r += blockDim.x) {
    const uint32_t hw_pos = cvt_sr_single<0>(v, r << 16) & 0xFu;
    const uint32_t hw_neg = cvt_sr_single<0>(-v, r << 16) & 0xFu;
    local += hw_pos != ref_e2m1_sr(v, r);
    local += hw_neg != ref_e2m1_sr(-v, r);
    // the accumulating form the quantizer uses: the code lands in the low nibble of the chosen byte, the other three
    // bytes of the destination are kept
    uint32_t acc = 0xA5C3F00Fu;
    cvt_sr_single_into<2>(acc, v, r << 16);
    local += ((acc >> 16) & 0xFu) != hw_pos || (acc & 0xFF00FFFFu) != 0xA500F00Fu;
    acc = 0x12345678u;
    cvt_sr_single_into<0>(acc, -v, r << 16);
    local += (acc & 0xFu) != hw_neg || (acc & 0xFFFFFF00u) != 0x12345600u;
  }
  if (local) atomicAdd(bad, local);
}

__global__ __launch_bounds__(256) void selftest_e4m3_kernel(unsigned long long* bad) {
  unsigned long long local = 0;
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  for (uint64_t w = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; w < 0x7F800000ull; w += stride) {
    const float u = __uint_as_float(static_cast<uint32_t>(w));
    const uint32_t code = e4m3_encode(u);
    local += code != ref_e4m3(u);
    local += (code < 0x7Fu) && (e4m3_decode(code) != __uint_as_float(
        (code >> 3) ? (((code >> 3) + 120u) << 23) | ((code & 7u) << 20) : __float_as_uint(static_cast<float>(code & 7u) * 0.001953125f)));
  }
  if (local) atomicAdd(bad, local);
}

// FP32 -> bf16 through the packed conversion instruction against the integer formulation of round-to-nearest-even,
// over every finite pattern (both halves of the pair).
__global__ __launch_bounds__(256) void selftest_bf16_kernel(unsigned long long* bad) {
  unsigned long long local = 0;
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  for (uint64_t w = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; w < 0x100000000ull; w += stride) {
    const uint32_t bits = static_cast<uint32_t>(w);
    if ((bits & 0x7F800000u) == 0x7F800000u) continue;     // Inf / NaN: outside the kernels' precondition
    const float x = __uint_as_float(bits);
    const float y = __uint_as_float(bits ^ 0x80000000u);
    local += f32x2_to_bf16(x, y) != (f32_to_bf16(x) | (f32_to_bf16(y) << 16));
  }
  if (local) atomicAdd(bad, local);
}

__global__ __launch_bounds__(256) void selftest_div6_kernel(unsigned long long* bad) {
  unsigned long long local = 0;
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  for (uint64_t w = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; w < 0x7F800000ull; w += stride) {
    const float x = __uint_as_float(static_cast<uint32_t>(w));
    local += __float_as_uint(div_by_6(x)) != __float_as_uint(x / 6.0f);
  }
  if (local) atomicAdd(bad, local);
}

}  // namespace

hipError_t run_selftest(uint64_t* mismatches_dev, hipStream_t s) {
  unsigned long long* dev = reinterpret_cast<unsigned long long*>(mismatches_dev);
  hipLaunchKernelGGL(selftest_rne_kernel, dim3(4096), dim3(256), 0, s, dev + 0);
  hipLaunchKernelGGL(selftest_sr_kernel, dim3(0x40E1u * 5u), dim3(256), 0, s, dev + 1);
  hipLaunchKernelGGL(selftest_e4m3_kernel, dim3(4096), dim3(256), 0, s, dev + 2);
  hipLaunchKernelGGL(selftest_div6_kernel, dim3(4096), dim3(256), 0, s, dev + 3);
  hipLaunchKernelGGL(selftest_bf16_kernel, dim3(4096), dim3(256), 0, s, dev + 4);
  return hipGetLastError();
}

}  // namespace nvfp4
