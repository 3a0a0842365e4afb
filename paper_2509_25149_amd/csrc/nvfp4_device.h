// Device-side helpers shared by the gfx950 kernels: number-format conversions,
// the Philox4x32-10 counter generator and the 16-point Hadamard butterfly.
// gfx950 only; wavefront size 64.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nvfp4 {

typedef float float2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// FP32 -> bf16, round to nearest even (finite inputs; NaN stays NaN).
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t w = __float_as_uint(f);
  if ((w & 0x7FFFFFFFu) > 0x7F800000u) return (w >> 16) | 0x40u;
  return (w + 0x7FFFu + ((w >> 16) & 1u)) >> 16;
}

// Two FP32 -> two bf16 in one dword (a in the low half), round to nearest even: the chip's packed conversion
// (v_cvt_pk_bf16_f32) instead of seven integer operations per value.
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16(float a, float b) {
  const float2v v = {a, b};
  union {
    bf16x2v h;
    uint32_t u;
  } c;
  c.h = __builtin_convertvector(v, bf16x2v);
  return c.u;
}

// Tensor-level encode / decode scale from the amax (App. B.1 Eq. 1).
__device__ __forceinline__ void tensor_scales(float amax, float& s_enc, float& s_dec) {
  if (amax == 0.0f) {
    s_enc = 1.0f;
  } else {
    s_enc = 2688.0f / amax;  // 6 * 448
    if (__builtin_isinf(s_enc)) s_enc = 3.4028234663852886e38f;
  }
  s_dec = 1.0f / s_enc;
}

// Non-negative FP32 -> E4M3 byte, RNE, saturating at 448 (App. B.2 Eq. 3).
// v_cvt_pk_fp8_f32 rounds to nearest even and returns NaN above the range, so
// the value is clamped first.
__device__ __forceinline__ uint32_t e4m3_encode(float u) {
  u = fminf(u, 448.0f);
  return static_cast<uint32_t>(__builtin_amdgcn_cvt_pk_fp8_f32(u, 0.0f, 0, false)) & 0xFFu;
}

__device__ __forceinline__ float e4m3_decode(uint32_t code) {
  return __builtin_amdgcn_cvt_f32_fp8(static_cast<int>(code), 0);
}

// x / 6 with IEEE round-to-nearest, for finite x >= 0, mostly without the
// hardware division sequence: one multiply by the rounded reciprocal, then one
// Newton-style correction with an exact FMA residual.  That is bit-identical to
// x / 6.0f for every x >= 2^-124 (below, the residual leaves the normal range);
// if any lane of the wavefront is below, the whole wavefront divides for real.
// Checked against IEEE division over all finite non-negative inputs by the
// self-test.  The result feeds the stored block scale of App. B.2 Eq. 2.
__device__ __forceinline__ float div_by_6(float x) {
  if (__builtin_amdgcn_ballot_w64(x < 0x1p-124f) != 0) return x / 6.0f;
  const float c = 0.16666667163372040f;           // RN(1/6)
  const float q = x * c;
  const float r = __builtin_fmaf(-q, 6.0f, x);     // exact residual x - 6q
  return __builtin_fmaf(r, c, q);
}

// Stored block scale and the "real" block encode scale (App. B.2):
//   code    = e4m3(amax_b / 6 * s_enc)
//   s_enc_b = 1 / (fp32(code) * s_dec), 0 when the stored scale is 0.
__device__ __forceinline__ float block_scale(float amax_b, float s_enc, float s_dec, uint32_t& code) {
  const float t = amax_b / 6.0f;
  code = e4m3_encode(t * s_enc);
  const float den = e4m3_decode(code) * s_dec;
  return den == 0.0f ? 0.0f : 1.0f / den;
}

// Two scaled values -> one byte of two E2M1 codes written into byte `kSel`
// of `old` (round to nearest even, saturating; matches the tie rule "even
// code").  The instruction's scale operand divides by a power of two only; it
// is held at 1.
template <int kSel>
__device__ __forceinline__ uint32_t cvt_rne_pair(uint32_t old, float v0, float v1) {
  return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(old, v0, v1, 1.0f, kSel);
}

// Stochastic rounding of one value with a 16-bit random integer placed in the
// top half of `rand_hi16`: the instruction adds the top 22 bits of its random
// operand below the kept mantissa bit, so with the low 16 bits clear it rounds
// up iff floor(p * 2^16) + r >= 2^16.  The result's only meaningful bits are
// the low nibble of byte `kSel`: the high nibble belongs to the pair's second
// value (which sees a rotated random word), and the other three bytes are
// whatever the destination register held -- this compiler does not tie the
// builtin's first operand to its result, so partial results cannot be chained
// through it and are merged with merge_bytes() instead.
template <int kSel>
__device__ __forceinline__ uint32_t cvt_sr_single(float v, uint32_t rand_hi16) {
  float2v p;   // the pair's second value is never looked at: it stays undefined so that no register move is spent on it
  p.x = v;
  return __builtin_amdgcn_cvt_scalef32_sr_pk_fp4_f32(0u, p, rand_hi16, 1.0f, kSel);
}

// The same conversion written into byte kSel of `acc`, the other three bytes kept: the instruction only writes the byte
// it is told to, but the builtin does not say so to the compiler (see above), so the accumulating form is spelled in
// assembly with the destination tied.  Four of these fill a dword without any merging.
template <int kSel>
__device__ __forceinline__ void cvt_sr_single_into(uint32_t& acc, float v, uint32_t rand_hi16) {
  float2v p;   // the pair's second value is never looked at
  p.x = v;
  asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,%3,%4]" : "+v"(acc) : "v"(p), "v"(rand_hi16), "n"(kSel & 1), "n"(kSel >> 1));
}

// (a & mask) | (b & ~mask) in one v_bitop3_b32 (truth table: the expression evaluated on
// a = 0xF0, b = 0xCC, mask = 0xAA).  Spelled with the builtin so that the compiler keeps it one
// instruction instead of re-deriving the nibble masks term by term.
__device__ __forceinline__ uint32_t bit_select(uint32_t mask, uint32_t a, uint32_t b) {
  return __builtin_amdgcn_bitop3_b32(a, b, mask, 0xE4);
}

// a ^ b ^ c in one instruction
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// byte t of the result is byte t of b[t]
__device__ __forceinline__ uint32_t merge_bytes(uint32_t b0, uint32_t b1, uint32_t b2, uint32_t b3) {
  return bit_select(0x0000FFFFu, bit_select(0x000000FFu, b0, b1), bit_select(0x00FF0000u, b2, b3));
}

// low nibbles of `even` and of `odd` interleaved: byte t = odd.nibble(2t) << 4 | even.nibble(2t)
__device__ __forceinline__ uint32_t interleave_nibbles(uint32_t even, uint32_t odd) {
  return bit_select(0x0F0F0F0Fu, even, odd << 4);
}

// Philox4x32-10 (Salmon et al., SC'11).
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = static_cast<uint64_t>(c0) * 0xD2511F53ull;
    const uint64_t p1 = static_cast<uint64_t>(c2) * 0xCD9E8D57ull;
    const uint32_t n0 = xor3(static_cast<uint32_t>(p1 >> 32), c1, k0);
    const uint32_t n2 = xor3(static_cast<uint32_t>(p0 >> 32), c3, k1);
    c1 = static_cast<uint32_t>(p1);
    c3 = static_cast<uint32_t>(p0);
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0;
  out[1] = c1;
  out[2] = c2;
  out[3] = c3;
}

// y = H16 (s .* v): sign diagonal, butterfly stages h = 1, 2, 4, 8 in this
// order, then the 1/4 normalisation (App. C).  Every add is one FP32 rounding.
__device__ __forceinline__ void rht16(float v[16], uint32_t sign_mask) {
#pragma unroll
  for (int i = 0; i < 16; ++i)
    v[i] = __uint_as_float(__float_as_uint(v[i]) ^ (((sign_mask >> i) & 1u) << 31));
#pragma unroll
  for (int h = 1; h < 16; h <<= 1) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if ((i & h) == 0) {
        const float a = v[i], b = v[i + h];
        v[i] = a + b;
        v[i + h] = a - b;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] *= 0.25f;
}

// x = s .* (H16 y)
__device__ __forceinline__ void rht16_inverse(float v[16], uint32_t sign_mask) {
  rht16(v, 0u);
#pragma unroll
  for (int i = 0; i < 16; ++i)
    v[i] = __uint_as_float(__float_as_uint(v[i]) ^ (((sign_mask >> i) & 1u) << 31));
}

// Value held by lane ^ 1 / lane ^ 2, through a DPP quad permutation (one VALU operation; the shuffle intrinsic goes
// through the LDS crossbar and has to be waited for).  All four lanes of a quad must be active.
__device__ __forceinline__ uint32_t lane_xor1(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1, 0, 3, 2]
}
__device__ __forceinline__ uint32_t lane_xor2(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2, 3, 0, 1]
}
__device__ __forceinline__ float lane_xor1(float v) { return __uint_as_float(lane_xor1(__float_as_uint(v))); }
__device__ __forceinline__ float lane_xor2(float v) { return __uint_as_float(lane_xor2(__float_as_uint(v))); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// 32-point transform of the MXFP4 mode (Sec. 5: rotation size 32 to match the block size; App. C):
// y = H32 (s .* v), butterfly stages h = 1, 2, 4, 8, 16, then one multiply by fl(1/sqrt(32)).
__device__ __forceinline__ void hadamard32(float v[32]) {
#pragma unroll
  for (int h = 1; h < 32; h <<= 1) {
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      if ((i & h) == 0) {
        const float a = v[i], b = v[i + h];
        v[i] = a + b;
        v[i + h] = a - b;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 32; ++i) v[i] = 0.176776695296636893f * v[i];
}

__device__ __forceinline__ void flip_signs32(float v[32], uint32_t sign_mask) {
#pragma unroll
  for (int i = 0; i < 32; ++i) v[i] = __uint_as_float(__float_as_uint(v[i]) ^ (((sign_mask >> i) & 1u) << 31));
}

__device__ __forceinline__ void rht32(float v[32], uint32_t sign_mask) {
  flip_signs32(v, sign_mask);
  hadamard32(v);
}

// H32 is symmetric and orthogonal: x = s .* (H32 y)
__device__ __forceinline__ void rht32_inverse(float y[32], uint32_t sign_mask) {
  hadamard32(y);
  flip_signs32(y, sign_mask);
}

// 2^(byte - 127) for a UE8M0 scale byte (Sec. 2), exact (byte 0 is the subnormal 2^-127)
__device__ __forceinline__ float ue8m0_decode(uint32_t byte) {
  return __uint_as_float(byte == 0u ? 0x00400000u : byte << 23);
}

}  // namespace nvfp4
