// NVFP4 -> FP32 / bf16 decode for gfx950: value(code) * block scale * s_dec
// (Sec. 2: decode with the reciprocal of the encode scale; App. B.2), with an
// optional inverse of the 16-point rotation of App. C.
#include "nvfp4_internal.h"
#include "nvfp4_device.h"

namespace nvfp4 {

namespace {

template <int kByte>
__device__ __forceinline__ void decode_pair_f32(uint32_t codes, float* out) {
  const float2v p = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, kByte);
  out[0] = p.x;
  out[1] = p.y;
}

template <bool kBf16Out>
__global__ __launch_bounds__(256) void dequantize_kernel(Operand q, int64_t K, bool undo_rht,
                                                         uint32_t sign_mask, void* __restrict__ outv,
                                                         int64_t ld_out) {
  const int64_t nblk = K / 16;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= q.outer * nblk) return;
  const int64_t o = idx / nblk, b = idx % nblk;
  const uint2 c = *reinterpret_cast<const uint2*>(q.codes + o * (K / 2) + b * 8);
  const float sd = e4m3_decode(q.scales[o * nblk + b]);
  const float s_dec = q.ts[q.ts_per_row ? o : 0];   // per tensor, or this row's own (App. B.1, last sentence)
  float v[16];
  decode_pair_f32<0>(c.x, v + 0);
  decode_pair_f32<1>(c.x, v + 2);
  decode_pair_f32<2>(c.x, v + 4);
  decode_pair_f32<3>(c.x, v + 6);
  decode_pair_f32<0>(c.y, v + 8);
  decode_pair_f32<1>(c.y, v + 10);
  decode_pair_f32<2>(c.y, v + 12);
  decode_pair_f32<3>(c.y, v + 14);
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const float t = v[k] * sd;
    v[k] = t * s_dec;
  }
  if (undo_rht) rht16_inverse(v, sign_mask);
  if (kBf16Out) {
    uint32_t w[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = f32x2_to_bf16(v[2 * k], v[2 * k + 1]);
    uint4* dst = reinterpret_cast<uint4*>(static_cast<uint16_t*>(outv) + o * ld_out + b * 16);
    dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
    dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
  } else {
    float4v* dst = reinterpret_cast<float4v*>(static_cast<float*>(outv) + o * ld_out + b * 16);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      float4v f;
      f[0] = v[4 * t];
      f[1] = v[4 * t + 1];
      f[2] = v[4 * t + 2];
      f[3] = v[4 * t + 3];
      dst[t] = f;
    }
  }
}

// MXFP4: one thread per 32-block, value(code) * 2^e (Sec. 2), optional inverse 32-point rotation.
template <bool kBf16Out>
__global__ __launch_bounds__(256) void dequantize_mx_kernel(Operand q, int64_t K, bool undo_rht, uint32_t sign_mask,
                                                            void* __restrict__ outv, int64_t ld_out) {
  const int64_t nblk = K / 32;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= q.outer * nblk) return;
  const int64_t o = idx / nblk, b = idx % nblk;
  const uint4 c = *reinterpret_cast<const uint4*>(q.codes + o * (K / 2) + b * 16);
  const float sd = ue8m0_decode(q.scales[o * nblk + b]);
  const uint32_t cw[4] = {c.x, c.y, c.z, c.w};
  float v[32];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    decode_pair_f32<0>(cw[t], v + 8 * t + 0);
    decode_pair_f32<1>(cw[t], v + 8 * t + 2);
    decode_pair_f32<2>(cw[t], v + 8 * t + 4);
    decode_pair_f32<3>(cw[t], v + 8 * t + 6);
  }
#pragma unroll
  for (int k = 0; k < 32; ++k) v[k] = v[k] * sd;
  if (undo_rht) rht32_inverse(v, sign_mask);
  if (kBf16Out) {
    uint4* dst = reinterpret_cast<uint4*>(static_cast<uint16_t*>(outv) + o * ld_out + b * 32);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      uint32_t w[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) w[k] = f32x2_to_bf16(v[8 * t + 2 * k], v[8 * t + 2 * k + 1]);
      dst[t] = make_uint4(w[0], w[1], w[2], w[3]);
    }
  } else {
    float4v* dst = reinterpret_cast<float4v*>(static_cast<float*>(outv) + o * ld_out + b * 32);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      float4v f;
      f[0] = v[4 * t];
      f[1] = v[4 * t + 1];
      f[2] = v[4 * t + 2];
      f[3] = v[4 * t + 3];
      dst[t] = f;
    }
  }
}

// NVFP4 with the inverse of a rotation of another size (2, 4, 32, 128 points; Sec. 4.2 "Hadamard matrix size"):
// one thread per max(16, d) elements.  x = s .* (H_d y) with the same stage order and single 1/sqrt(d) multiply as
// the forward transform (H_d is symmetric and orthogonal, App. C).
template <bool kBf16Out, int kD>
__global__ __launch_bounds__(256) void dequantize_rot_kernel(Operand q, int64_t K, uint4 sign_words, void* __restrict__ outv,
                                                             int64_t ld_out) {
  constexpr int kE = kD < 16 ? 16 : kD;   // elements per thread
  const int64_t nper = K / kE;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= q.outer * nper) return;
  const int64_t o = idx / nper, b = idx % nper;
  const float s_dec = q.ts[q.ts_per_row ? o : 0];
  float v[kE];
#pragma unroll
  for (int blk = 0; blk < kE / 16; ++blk) {
    const uint2 c = *reinterpret_cast<const uint2*>(q.codes + o * (K / 2) + b * (kE / 2) + blk * 8);
    const float sd = e4m3_decode(q.scales[o * (K / 16) + b * (kE / 16) + blk]);
    float* w = v + 16 * blk;
    decode_pair_f32<0>(c.x, w + 0);
    decode_pair_f32<1>(c.x, w + 2);
    decode_pair_f32<2>(c.x, w + 4);
    decode_pair_f32<3>(c.x, w + 6);
    decode_pair_f32<0>(c.y, w + 8);
    decode_pair_f32<1>(c.y, w + 10);
    decode_pair_f32<2>(c.y, w + 12);
    decode_pair_f32<3>(c.y, w + 14);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const float t = w[k] * sd;
      w[k] = t * s_dec;
    }
  }
#pragma unroll
  for (int h = 1; h < kD; h <<= 1) {
#pragma unroll
    for (int i = 0; i < kE; ++i) {
      if ((i & h) == 0) {
        const float a = v[i], c = v[i + h];
        v[i] = a + c;
        v[i + h] = a - c;
      }
    }
  }
  constexpr float kNorm = kD == 2 ? 0.707106781186547524f : kD == 4 ? 0.5f : kD == 32 ? 0.176776695296636893f : 0.0883883476483184405f;
  const uint32_t sw[4] = {sign_words.x, sign_words.y, sign_words.z, sign_words.w};
#pragma unroll
  for (int i = 0; i < kE; ++i) {
    const int bit = i % kD;
    v[i] = __uint_as_float(__float_as_uint(kNorm * v[i]) ^ (((sw[bit >> 5] >> (bit & 31)) & 1u) << 31));
  }
  if (kBf16Out) {
    uint4* dst = reinterpret_cast<uint4*>(static_cast<uint16_t*>(outv) + o * ld_out + b * kE);
#pragma unroll
    for (int t = 0; t < kE / 8; ++t) {
      uint32_t w[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) w[k] = f32x2_to_bf16(v[8 * t + 2 * k], v[8 * t + 2 * k + 1]);
      dst[t] = make_uint4(w[0], w[1], w[2], w[3]);
    }
  } else {
    float4v* dst = reinterpret_cast<float4v*>(static_cast<float*>(outv) + o * ld_out + b * kE);
#pragma unroll
    for (int t = 0; t < kE / 4; ++t) {
      float4v f;
      f[0] = v[4 * t];
      f[1] = v[4 * t + 1];
      f[2] = v[4 * t + 2];
      f[3] = v[4 * t + 3];
      dst[t] = f;
    }
  }
}

template <int kD>
void launch_rot(const DequantArgs& d, hipStream_t s) {
  const int64_t total = d.q.outer * (d.K / (kD < 16 ? 16 : kD));
  const dim3 grid(static_cast<unsigned>((total + 255) / 256));
  const uint4 signs = make_uint4(d.sign_words[0], d.sign_words[1], d.sign_words[2], d.sign_words[3]);
  if (d.out_bf16)
    hipLaunchKernelGGL((dequantize_rot_kernel<true, kD>), grid, dim3(256), 0, s, d.q, d.K, signs, d.out, d.ld_out);
  else
    hipLaunchKernelGGL((dequantize_rot_kernel<false, kD>), grid, dim3(256), 0, s, d.q, d.K, signs, d.out, d.ld_out);
}

}  // namespace

hipError_t launch_dequantize_mx(const DequantArgs& d, hipStream_t s) {
  const int64_t total = d.q.outer * (d.K / 32);
  if (total == 0) return hipSuccess;
  const dim3 grid(static_cast<unsigned>((total + 255) / 256));
  if (d.out_bf16)
    hipLaunchKernelGGL(dequantize_mx_kernel<true>, grid, dim3(256), 0, s, d.q, d.K, d.undo_rht, d.sign_mask, d.out, d.ld_out);
  else
    hipLaunchKernelGGL(dequantize_mx_kernel<false>, grid, dim3(256), 0, s, d.q, d.K, d.undo_rht, d.sign_mask, d.out, d.ld_out);
  return hipGetLastError();
}

hipError_t launch_dequantize(const DequantArgs& d, hipStream_t s) {
  const int64_t total = d.q.outer * (d.K / 16);
  if (total == 0) return hipSuccess;
  if (d.undo_rht && d.rht_dim != 16) {
    switch (d.rht_dim) {
      case 2: launch_rot<2>(d, s); break;
      case 4: launch_rot<4>(d, s); break;
      case 32: launch_rot<32>(d, s); break;
      case 128: launch_rot<128>(d, s); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  const dim3 grid(static_cast<unsigned>((total + 255) / 256));
  if (d.out_bf16)
    hipLaunchKernelGGL(dequantize_kernel<true>, grid, dim3(256), 0, s, d.q, d.K, d.undo_rht, d.sign_mask, d.out, d.ld_out);
  else
    hipLaunchKernelGGL(dequantize_kernel<false>, grid, dim3(256), 0, s, d.q, d.K, d.undo_rht, d.sign_mask, d.out, d.ld_out);
  return hipGetLastError();
}

}  // namespace nvfp4
