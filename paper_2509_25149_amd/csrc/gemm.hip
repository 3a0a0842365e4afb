// NVFP4 block-scaled GEMM for gfx950 (Sec. 2 "Hardware support via Tensor
// Cores"; App. B.3 Eq. 5):
//   D[m, n] = s_dec^A s_dec^B  sum_b sA[m,b] sB[n,b]  sum_{k in b} A[m,k] B[n,k]
//
// How the scales are applied on CDNA4.  The chip's scaled MFMA takes one
// power-of-two (E8M0) scale per 32 elements; NVFP4 has an E4M3 scale per 16.
// An E2M1 value (2 significant bits) times an E4M3 scale (4 significant
// bits) needs up to 6 significant bits, which FP8 (4 bits) cannot hold, so
// a decode to FP8 would already break the 1e-5 accuracy target.  FP16 holds
// the product exactly (11 bits; range 2^-10 .. 2688 is inside FP16's normal
// range), so each operand tile is decoded ONCE per workgroup to
// value * block_scale in FP16 while it is staged into LDS, and the
// contraction runs on v_mfma_f32_32x32x16_f16: every product is exact and the
// accumulation is FP32, which is Eq. 5 up to FP32 summation order.  The two
// tensor-level decode scales are applied to the finished sums.
#include "nvfp4_internal.h"
#include "nvfp4_device.h"

namespace nvfp4 {

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_LD = BK + 8;  // halfs per LDS row; the 16-byte pad keeps 128-bit reads conflict free
constexpr int kGemmThreads = 256;

template <int kByte>
__device__ __forceinline__ half2v decode_pair(uint32_t codes, half2v scale) {
  return __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, kByte) * scale;
}

// 8 codes (one dword) -> 8 FP16 values, each value * block scale.
__device__ __forceinline__ uint4 decode8(uint32_t codes, half2v scale) {
  union {
    half2v h[4];
    uint4 u;
  } o;
  o.h[0] = decode_pair<0>(codes, scale);
  o.h[1] = decode_pair<1>(codes, scale);
  o.h[2] = decode_pair<2>(codes, scale);
  o.h[3] = decode_pair<3>(codes, scale);
  return o.u;
}

__device__ __forceinline__ half2v scale_to_half2(uint32_t e4m3_byte) {
  const _Float16 s = static_cast<_Float16>(e4m3_decode(e4m3_byte));  // exact: 4 significant bits
  half2v r;
  r.x = s;
  r.y = s;
  return r;
}

// Stage 32 elements (two 16-blocks) of one operand row into LDS as FP16.
__device__ __forceinline__ void stage_row(const Operand& op, int64_t K, int64_t row, int64_t k,
                                          _Float16* lds_row) {
  uint2 c01 = make_uint2(0u, 0u), c23 = make_uint2(0u, 0u);
  uint32_t s0 = 0, s1 = 0;
  if (row < op.outer) {
    const uint8_t* cp = op.codes + row * (K / 2) + k / 2;
    const uint8_t* sp = op.scales + row * (K / 16) + k / 16;
    if (k < K) {
      c01 = *reinterpret_cast<const uint2*>(cp);
      s0 = sp[0];
    }
    if (k + 16 < K) {
      c23 = *reinterpret_cast<const uint2*>(cp + 8);
      s1 = sp[1];
    }
  }
  const half2v h0 = scale_to_half2(s0), h1 = scale_to_half2(s1);
  uint4* dst = reinterpret_cast<uint4*>(lds_row);
  dst[0] = decode8(c01.x, h0);
  dst[1] = decode8(c01.y, h0);
  dst[2] = decode8(c23.x, h1);
  dst[3] = decode8(c23.y, h1);
}

template <bool kBf16Out>
__global__ __launch_bounds__(kGemmThreads) void gemm_kernel(Operand A, Operand B, int64_t K,
                                                            void* __restrict__ Dv, int64_t ldd) {
  __shared__ __attribute__((aligned(16))) _Float16 As[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) _Float16 Bs[BN * LDS_LD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;  // 2 x 2 wavefronts, 64 x 64 outputs each
  const int64_t m0 = static_cast<int64_t>(blockIdx.y) * BM, n0 = static_cast<int64_t>(blockIdx.x) * BN;

  // acc[i][j]: 32x32 block with n-rows (B operand rows) as the MFMA's M index
  // and m-rows as its N index, so a lane ends up with 4 consecutive n.
  float16v acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int srow = tid >> 1, shalf = tid & 1;
  const int l32 = lane & 31, kq = (lane >> 5) * 8;

  for (int64_t k0 = 0; k0 < K; k0 += BK) {
    stage_row(A, K, m0 + srow, k0 + shalf * 32, As + srow * LDS_LD + shalf * 32);
    stage_row(B, K, n0 + srow, k0 + shalf * 32, Bs + srow * LDS_LD + shalf * 32);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      half8v af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = *reinterpret_cast<const half8v*>(As + (wm * 64 + i * 32 + l32) * LDS_LD + kk + kq);
        bf[i] = *reinterpret_cast<const half8v*>(Bs + (wn * 64 + i * 32 + l32) * LDS_LD + kk + kq);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[j], af[i], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // Tensor-level decode scales on the finished sums (App. B.3, after Eq. 5).
  const float out_scale = A.ts[0] * B.ts[0];
  const int M = static_cast<int>(A.outer - m0 < BM ? A.outer - m0 : BM);
  const int N = static_cast<int>(B.outer - n0 < BN ? B.outer - n0 : BN);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = wm * 64 + i * 32 + l32;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = wn * 64 + j * 32 + q * 8 + (lane >> 5) * 4;
        if (m < M && n < N) {  // N is a multiple of 16, so the 4 columns are in or out together
          float4v v;
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] = acc[i][j][q * 4 + t] * out_scale;
          if (kBf16Out) {
            uint16_t* d = static_cast<uint16_t*>(Dv) + (m0 + m) * ldd + n0 + n;
            uint2 o;
            o.x = f32_to_bf16(v[0]) | (f32_to_bf16(v[1]) << 16);
            o.y = f32_to_bf16(v[2]) | (f32_to_bf16(v[3]) << 16);
            *reinterpret_cast<uint2*>(d) = o;
          } else {
            float* d = static_cast<float*>(Dv) + (m0 + m) * ldd + n0 + n;
            *reinterpret_cast<float4v*>(d) = v;
          }
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  const dim3 grid(static_cast<unsigned>((g.b.outer + BN - 1) / BN), static_cast<unsigned>((g.a.outer + BM - 1) / BM));
  if (g.out_bf16)
    hipLaunchKernelGGL(gemm_kernel<true>, grid, dim3(kGemmThreads), 0, s, g.a, g.b, g.K, g.d, g.ldd);
  else
    hipLaunchKernelGGL(gemm_kernel<false>, grid, dim3(kGemmThreads), 0, s, g.a, g.b, g.K, g.d, g.ldd);
  return hipGetLastError();
}

}  // namespace nvfp4
