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
#include "gemm_epilogue.h"

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
                                                            void* __restrict__ Dv, int64_t ldd, bool accumulate) {
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
  const TensorScales ts{A.ts, B.ts, A.ts_per_row != 0, B.ts_per_row != 0};
  const bool vec = ts.a_per_row || ts.b_per_row;
  const float out_scale = vec ? 0.0f : A.ts[0] * B.ts[0];
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
          const float4v sc = scale4(ts, out_scale, vec, true, m0 + m, n0 + n);
          float4v v;
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] = acc[i][j][q * 4 + t] * sc[t];
          if (kBf16Out) {
            uint16_t* d = static_cast<uint16_t*>(Dv) + (m0 + m) * ldd + n0 + n;
            uint2 o;
            o.x = f32x2_to_bf16(v[0], v[1]);
            o.y = f32x2_to_bf16(v[2], v[3]);
            *reinterpret_cast<uint2*>(d) = o;
          } else {
            float* d = static_cast<float*>(Dv) + (m0 + m) * ldd + n0 + n;
            if (accumulate) v += *reinterpret_cast<const float4v*>(d);
            *reinterpret_cast<float4v*>(d) = v;
          }
        }
      }
    }
  }
}


// ---------------------------------------------------------------- large-tile kernel
// 256 x 256 outputs per workgroup, K step 64, 512 threads = 8 wavefronts in a
// 2 (m) x 4 (n) grid, each owning 128 x 64 outputs as 8 x 4 MFMA 16x16 blocks
// (128 accumulator registers per lane).  The decoded FP16 tiles are
// double-buffered in LDS (2 x 64 KiB), one barrier per K step.
//
// The two halves of the workgroup run the step's two phases in opposite
// order ("ping-pong"): wavefronts 0-3 (one per SIMD) issue their global loads,
// run the step's 64 MFMAs and then decode the NEXT A tile into the other LDS
// buffer; wavefronts 4-7 first decode the next B tile, then issue their loads
// for the step after and run their MFMAs.  On every SIMD one wavefront is
// therefore in its VALU/LDS-write phase while the other keeps the matrix pipe
// busy.  Inside the MFMA phase the fragments of sub-step kk+1 are read from LDS
// before the MFMAs of sub-step kk are issued.
//
// LDS layout: one row = 64 FP16 = eight 16-byte chunks, no padding; chunk c of
// row r is stored at chunk position c ^ ((r >> 1) & 7).  With a 128-byte row
// stride, 16 consecutive rows reading the same logical chunk then touch 16
// different 16-byte bank groups, and the staging writes are conflict free too.
constexpr int TM = 256, TN = 256, TK = 64;
constexpr int kBigThreads = 512;
constexpr int kRowBytes = TK * 2;                         // 128
constexpr int kOperandBytes = TM * kRowBytes;              // 32 KiB per operand tile
constexpr int kStageBytes = 2 * kOperandBytes;             // 64 KiB

__device__ __forceinline__ int swz(int row, int chunk) { return row * kRowBytes + ((chunk ^ ((row >> 1) & 7)) << 4); }

struct Prefetch {
  uint4 lo, hi;     // 64 codes of one row
  uint32_t scales;  // four E4M3 bytes
};

__device__ __forceinline__ void fetch_row(Prefetch& p, const Operand& op, int64_t K, int64_t row, int64_t k) {
  p.lo = make_uint4(0u, 0u, 0u, 0u);
  p.hi = make_uint4(0u, 0u, 0u, 0u);
  p.scales = 0u;
  if (row < op.outer) {
    const uint4* c = reinterpret_cast<const uint4*>(op.codes + row * (K / 2) + k / 2);
    p.lo = c[0];
    p.hi = c[1];
    p.scales = *reinterpret_cast<const uint32_t*>(op.scales + row * (K / 16) + k / 16);
  }
}

__device__ __forceinline__ void stage_decoded(const Prefetch& p, char* tile, int row) {
  const half2v h0 = scale_to_half2(p.scales & 0xFFu), h1 = scale_to_half2((p.scales >> 8) & 0xFFu);
  const half2v h2 = scale_to_half2((p.scales >> 16) & 0xFFu), h3 = scale_to_half2(p.scales >> 24);
  *reinterpret_cast<uint4*>(tile + swz(row, 0)) = decode8(p.lo.x, h0);
  *reinterpret_cast<uint4*>(tile + swz(row, 1)) = decode8(p.lo.y, h0);
  *reinterpret_cast<uint4*>(tile + swz(row, 2)) = decode8(p.lo.z, h1);
  *reinterpret_cast<uint4*>(tile + swz(row, 3)) = decode8(p.lo.w, h1);
  *reinterpret_cast<uint4*>(tile + swz(row, 4)) = decode8(p.hi.x, h2);
  *reinterpret_cast<uint4*>(tile + swz(row, 5)) = decode8(p.hi.y, h2);
  *reinterpret_cast<uint4*>(tile + swz(row, 6)) = decode8(p.hi.z, h3);
  *reinterpret_cast<uint4*>(tile + swz(row, 7)) = decode8(p.hi.w, h3);
}

// Fragments of one 32-wide half of a K step for a 128 x 64 wave tile.  A 16x16x32 MFMA operand is
// 16 rows x 32 k: lane l holds the 8 consecutive k of 16-byte chunk (l >> 4) of row (l & 15).
// (16x16x32 rather than 32x32x16: more flop/s under the chip's power limit on the same operands.)
struct Frags {
  half8v a[8], b[4];
};

// `chunk` = half * 4 + (lane >> 4): the lane's 16-byte chunk of the 128-byte tile row.
__device__ __forceinline__ void load_frags(Frags& f, const char* at, const char* bt, int arow, int brow, int chunk) {
#pragma unroll
  for (int i = 0; i < 8; ++i) f.a[i] = *reinterpret_cast<const half8v*>(at + swz(arow + i * 16, chunk));
#pragma unroll
  for (int j = 0; j < 4; ++j) f.b[j] = *reinterpret_cast<const half8v*>(bt + swz(brow + j * 16, chunk));
}

// The MFMA's M index is the B row (n), its N index the A row (m): lane l ends up with the 4
// consecutive n = (l >> 4) * 4 .. + 3 of m = l & 15.
__device__ __forceinline__ void mma_step(float4v (&acc)[8][4], const Frags& f) {
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(f.b[j], f.a[i], acc[i][j], 0, 0, 0);
}

// The 64 MFMAs of one K step.
__device__ __forceinline__ void mma_tile(float4v (&acc)[8][4], const char* at, const char* bt, int arow, int brow,
                                         int lq) {
  Frags f0, f1;
  load_frags(f0, at, bt, arow, brow, 0 + lq);
  load_frags(f1, at, bt, arow, brow, 4 + lq);
  mma_step(acc, f0);
  mma_step(acc, f1);
}

template <bool kBf16Out>
__global__ __launch_bounds__(kBigThreads) void gemm_kernel_256(Operand A, Operand B, int64_t K,
                                                               void* __restrict__ Dv, int64_t ldd, bool accumulate,
                                                               int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) char lds[];

  // Workgroup -> output tile.  Consecutive workgroup ids land on different XCDs
  // (round robin over 8), each with its own L2: give every XCD a contiguous
  // range of tiles, walked in bands of 8 tile-rows so that the A and B panels a
  // band touches stay L2 resident.
  const int num_tiles = tiles_m * tiles_n;
  int pid = blockIdx.x;
  if ((num_tiles & 7) == 0) pid = (pid & 7) * (num_tiles >> 3) + (pid >> 3);
  constexpr int kBand = 8;
  const int band = pid / (kBand * tiles_n);
  const int band_rows = min(kBand, tiles_m - band * kBand);
  const int in_band = pid - band * kBand * tiles_n;
  const int tm = band * kBand + in_band % band_rows;
  const int tn = in_band / band_rows;
  const int64_t m0 = static_cast<int64_t>(tm) * TM, n0 = static_cast<int64_t>(tn) * TN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int group = wave >> 2;           // 0: stages A, MFMA first; 1: stages B, decode first
  const int wm = wave >> 2, wn = wave & 3;
  const int l16 = lane & 15, lq = lane >> 4;
  const int srow = tid & 255;            // the operand-tile row this thread stages
  const int arow = wm * 128 + l16, brow = wn * 64 + l16;

  float4v acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

  const Operand& mine = group == 0 ? A : B;
  const int64_t my_row = (group == 0 ? m0 : n0) + srow;
  const int my_off = group == 0 ? 0 : kOperandBytes;
  const int KT = static_cast<int>(K / TK);

  // Schedule per K step t (S = decode + store to LDS, M = the step's MFMAs, | = barrier):
  //   wavefronts 0-3:  M(t) S_A(t+1) | M(t+1) S_A(t+2) | ...
  //   wavefronts 4-7:  S_B(t+1) M(t) | S_B(t+2) M(t+1) | ...
  // written as one loop body  "fetch; M(t); [group 0: S(t+1)]; barrier; [group 1: S(t+2)]".
  Prefetch cur, nxt;
  fetch_row(cur, mine, K, my_row, 0);
  stage_decoded(cur, lds + my_off, srow);
  if (group == 1 && KT > 1) {
    fetch_row(cur, mine, K, my_row, TK);
    stage_decoded(cur, lds + kStageBytes + my_off, srow);
  }
  // Global loads run two K steps ahead of their decode, so the decode never waits on memory.
  if (1 + group < KT) fetch_row(cur, mine, K, my_row, static_cast<int64_t>(1 + group) * TK);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const char* tile = lds + (kt & 1) * kStageBytes;
    const int ahead = kt + 1 + group;    // the K step this wavefront stages during step kt
    if (ahead + 1 < KT) fetch_row(nxt, mine, K, my_row, static_cast<int64_t>(ahead + 1) * TK);
    mma_tile(acc, tile, tile + kOperandBytes, arow, brow, lq);
    if (group == 0 && ahead < KT) stage_decoded(cur, lds + (ahead & 1) * kStageBytes + my_off, srow);
    __syncthreads();
    if (group == 1 && ahead < KT) stage_decoded(cur, lds + (ahead & 1) * kStageBytes + my_off, srow);
    cur = nxt;
  }

  const TensorScales ts{A.ts, B.ts, A.ts_per_row != 0, B.ts_per_row != 0};
  const bool vec = ts.a_per_row || ts.b_per_row;
  const float out_scale = vec ? 0.0f : A.ts[0] * B.ts[0];
  const int M = static_cast<int>(A.outer - m0 < TM ? A.outer - m0 : TM);
  const int N = static_cast<int>(B.outer - n0 < TN ? B.outer - n0 : TN);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int m = wm * 128 + i * 16 + l16;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = wn * 64 + j * 16 + lq * 4;
      if (m < M && n < N) {  // N is a multiple of 16, so the 4 columns are in or out together
        float4v v = acc[i][j] * scale4(ts, out_scale, vec, true, m0 + m, n0 + n);
        if (kBf16Out) {
          uint16_t* d = static_cast<uint16_t*>(Dv) + (m0 + m) * ldd + n0 + n;
          uint2 o;
          o.x = f32x2_to_bf16(v[0], v[1]);
          o.y = f32x2_to_bf16(v[2], v[3]);
          *reinterpret_cast<uint2*>(d) = o;
        } else {
          float* d = static_cast<float*>(Dv) + (m0 + m) * ldd + n0 + n;
          if (accumulate) v += *reinterpret_cast<const float4v*>(d);
          *reinterpret_cast<float4v*>(d) = v;
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  // With a workspace: decode pass + FP16 GEMM (faster).  Without: the fused kernels below.
  if (gemm_two_pass_usable(g)) return launch_gemm_two_pass(g, s);
  // The large-tile kernel needs whole K steps of 64 and 16-byte aligned code rows.
  const bool big = (g.K % TK == 0) && (reinterpret_cast<uintptr_t>(g.a.codes) % 16 == 0) &&
                   (reinterpret_cast<uintptr_t>(g.b.codes) % 16 == 0);
  if (big) {
    static PerDeviceOnce once_bf16, once_f32;
    const hipError_t e = g.out_bf16 ? ensure_dynamic_lds(reinterpret_cast<const void*>(&gemm_kernel_256<true>), 2 * kStageBytes, once_bf16)
                                    : ensure_dynamic_lds(reinterpret_cast<const void*>(&gemm_kernel_256<false>), 2 * kStageBytes, once_f32);
    if (e != hipSuccess) return e;
    const int tiles_m = static_cast<int>((g.a.outer + TM - 1) / TM), tiles_n = static_cast<int>((g.b.outer + TN - 1) / TN);
    const dim3 grid(static_cast<unsigned>(tiles_m * tiles_n));
    if (g.out_bf16)
      hipLaunchKernelGGL(gemm_kernel_256<true>, grid, dim3(kBigThreads), 2 * kStageBytes, s, g.a, g.b, g.K, g.d, g.ldd, g.accumulate, tiles_m, tiles_n);
    else
      hipLaunchKernelGGL(gemm_kernel_256<false>, grid, dim3(kBigThreads), 2 * kStageBytes, s, g.a, g.b, g.K, g.d, g.ldd, g.accumulate, tiles_m, tiles_n);
    return hipGetLastError();
  }
  const dim3 grid(static_cast<unsigned>((g.b.outer + BN - 1) / BN), static_cast<unsigned>((g.a.outer + BM - 1) / BM));
  if (g.out_bf16)
    hipLaunchKernelGGL(gemm_kernel<true>, grid, dim3(kGemmThreads), 0, s, g.a, g.b, g.K, g.d, g.ldd, g.accumulate);
  else
    hipLaunchKernelGGL(gemm_kernel<false>, grid, dim3(kGemmThreads), 0, s, g.a, g.b, g.K, g.d, g.ldd, g.accumulate);
  return hipGetLastError();
}

}  // namespace nvfp4
