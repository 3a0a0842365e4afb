// MXFP4 GEMM for gfx950 on the block-scaled matrix instruction: the paper's
// comparison format (Sec. 2: E2M1 elements, one UE8M0 power-of-two scale per 32)
// is exactly what v_mfma_scale_f32_16x16x128_f8f6f4 consumes, so -- unlike the
// NVFP4 GEMM, whose E4M3-per-16 scales force a decode to FP16 -- the packed codes
// go from global memory through LDS into the matrix pipe untouched:
//   D[m, n] = sum_b 2^(ea[m,b] + eb[n,b]) sum_{k in b} A[m,k] B[n,k],  FP32 accumulation.
//
// Operand layout of the instruction with FP4 inputs (checked on the device):
// lane l carries row (l & 15) and the 32 consecutive k of block (l >> 4) as 16
// bytes (element 2t in the low nibble of byte t -- the storage format as it is)
// plus that block's scale byte; the 16x16 result puts D[(l >> 4) * 4 + i][l & 15]
// in register i of lane l, rows taken from the first operand.
//
// 256 x 256 outputs per workgroup, K step 128 (one instruction deep), 512 threads
// = 8 wavefronts (2 x 4) of 128 x 64.  LDS holds four stages of (A codes, B codes,
// A scales, B scales) = 34 KiB each (two K steps per barrier), filled by direct global->LDS loads: a code
// row of a stage is 64 bytes, so 16 consecutive tile rows are 1 KiB of LDS and a
// fragment read (16 rows x 4 blocks x 16 bytes) is one contiguous KiB.
#include "nvfp4_internal.h"
#include "nvfp4_device.h"

namespace nvfp4 {

namespace {

constexpr int TM = 256, TN = 256, TK = 128;
constexpr int kThreads = 512;
constexpr int kCodeRowBytes = TK / 2;                 // 64
constexpr int kCodeBytes = TM * kCodeRowBytes;        // 16 KiB per operand
constexpr int kScaleBytes = TM * (TK / 32);           // 1 KiB per operand
constexpr int kStageBytes = 2 * kCodeBytes + 2 * kScaleBytes;

typedef int int8v __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lds_ptr;

// 64 lanes x 16 (or 4) bytes from global memory straight into consecutive LDS at the wave-uniform
// LDS byte offset lds_off (global_load_lds_*; M0 carries the LDS address).  Inline assembly on
// purpose: for the builtin form the compiler makes every later LDS read wait for all direct loads
// in flight (it cannot tell the stages apart), which serialises the prefetch of the next stages
// with the reads of the current one.  The loop keeps them apart itself: s_waitcnt vmcnt(0) and a
// barrier stand between a stage's loads and its first read.
__device__ __forceinline__ void load16_to_lds(const uint8_t* src, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_off), "v"(src) : "memory", "m0");
}
__device__ __forceinline__ void load4_to_lds(const uint8_t* src, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" : : "s"(lds_off), "v"(src) : "memory", "m0");
}

// One operand fragment: the low four dwords are the 32 codes of the lane's block; the
// instruction ignores the rest of the 256-bit operand for FP4, so it is left undefined.
__device__ __forceinline__ int8v load_frag(const char* codes, int row, int kb) {
  const uint4 q = *reinterpret_cast<const uint4*>(codes + row * kCodeRowBytes + kb * 16);
  int8v f;
  f[0] = static_cast<int>(q.x);
  f[1] = static_cast<int>(q.y);
  f[2] = static_cast<int>(q.z);
  f[3] = static_cast<int>(q.w);
  return f;
}

template <bool kBf16Out>
__global__ __launch_bounds__(kThreads) void gemm_mx_kernel(Operand A, Operand B, int64_t K, void* __restrict__ Dv,
                                                           int64_t ldd, bool accumulate, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) char lds[];

  // Workgroup -> tile: consecutive ids go to different XCDs (round robin over 8, one L2 each);
  // every XCD gets a contiguous range of tiles, walked in bands of 8 tile rows.
  const int num_tiles = tiles_m * tiles_n;
  int pid = blockIdx.x;
  if ((num_tiles & 7) == 0) pid = (pid & 7) * (num_tiles >> 3) + (pid >> 3);
  constexpr int kBand = 8;
  const int band = pid / (kBand * tiles_n);
  const int band_rows = min(kBand, tiles_m - band * kBand);
  const int in_band = pid - band * kBand * tiles_n;
  const int tm = band * kBand + in_band % band_rows, tn = in_band / band_rows;
  const int64_t m0 = static_cast<int64_t>(tm) * TM, n0 = static_cast<int64_t>(tn) * TN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3, l16 = lane & 15, kb = lane >> 4;
  const int arow = wm * 128 + l16, brow = wn * 64 + l16;
  const int64_t code_ld = K / 2, scale_ld = K / 32;

  // Direct-load sources.  Codes: an instruction fills 16 tile rows (lane -> row lane / 4, 16-byte
  // piece lane % 4); every wavefront loads 32 rows of A and 32 rows of B.  Scales: an instruction
  // fills 64 tile rows x 4 bytes; wavefronts 0-3 take A, 4-7 take B.  Rows past the end of an
  // operand are clamped; they only feed outputs that are never stored.
  const uint8_t* ga[2];
  const uint8_t* gb[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int r = (wave * 2 + q) * 16 + (lane >> 2);
    ga[q] = A.codes + min<int64_t>(m0 + r, A.outer - 1) * code_ld + (lane & 3) * 16;
    gb[q] = B.codes + min<int64_t>(n0 + r, B.outer - 1) * code_ld + (lane & 3) * 16;
  }
  const int srow = (wave & 3) * 64 + lane;
  const uint8_t* gs = wave < 4 ? A.scales + min<int64_t>(m0 + srow, A.outer - 1) * scale_ld
                               : B.scales + min<int64_t>(n0 + srow, B.outer - 1) * scale_ld;
  const int s_off = 2 * kCodeBytes + (wave < 4 ? 0 : kScaleBytes) + (wave & 3) * 256;

  const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr)lds));
  auto issue = [&](int kt, int stage) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base + stage * kStageBytes);
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      load16_to_lds(ga[q] + static_cast<int64_t>(kt) * kCodeRowBytes, base + (wave * 2 + q) * 1024);
      load16_to_lds(gb[q] + static_cast<int64_t>(kt) * kCodeRowBytes, base + kCodeBytes + (wave * 2 + q) * 1024);
    }
    load4_to_lds(gs + static_cast<int64_t>(kt) * 4, base + s_off);
  };

  float4v acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

  // Fragment groups: a stage is two groups of (4 A fragments x 4 B fragments) = 16 MFMAs; the
  // fragments of the next group are requested from LDS before the MFMAs of the current one start.
  struct AFr {
    int8v f[4];
    int s[4];
  };
  struct BFr {
    int8v f[4];
    int s[4];
  };
  auto load_a = [&](AFr& a, const char* cur, int h) {
    const uint8_t* sc = reinterpret_cast<const uint8_t*>(cur + 2 * kCodeBytes);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a.f[i] = load_frag(cur, arow + (h * 4 + i) * 16, kb);
      a.s[i] = sc[(arow + (h * 4 + i) * 16) * 4 + kb];
    }
  };
  auto load_b = [&](BFr& b, const char* cur) {
    const uint8_t* sc = reinterpret_cast<const uint8_t*>(cur + 2 * kCodeBytes + kScaleBytes);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      b.f[j] = load_frag(cur + kCodeBytes, brow + j * 16, kb);
      b.s[j] = sc[(brow + j * 16) * 4 + kb];
    }
  };
  // The instruction's first operand supplies the rows of its result: passing B first leaves a lane
  // with 4 consecutive n of one m, which makes the output stores 64/128-bit.
  auto mma = [&](const AFr& a, const BFr& b, int h) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[h * 4 + i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b.f[j], a.f[i], acc[h * 4 + i][j], 4, 4, 0,
                                                                             b.s[j], 0, a.s[i]);
  };

  // Two K steps per barrier: LDS holds two buffers of two stages each (4 x 34 KiB); the loads of
  // the next pair of steps are in flight while this pair is multiplied.
  const int KT = static_cast<int>(K / TK);
  issue(0, 0);
  if (KT > 1) issue(1, 1);
  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): the direct loads have landed in LDS
  __syncthreads();

  int kt = 0;
  for (; kt + 1 < KT; kt += 2) {
    const int buf = (kt >> 1) & 1;
    if (kt + 2 < KT) issue(kt + 2, (buf ^ 1) * 2);
    if (kt + 3 < KT) issue(kt + 3, (buf ^ 1) * 2 + 1);
    const char* s0 = lds + (buf * 2) * kStageBytes;
    const char* s1 = s0 + kStageBytes;
    AFr a0, a1;
    BFr b0, b1;
    load_b(b0, s0);
    load_a(a0, s0, 0);
    __builtin_amdgcn_sched_barrier(0);
    load_a(a1, s0, 1);
    __builtin_amdgcn_sched_barrier(0);
    mma(a0, b0, 0);
    __builtin_amdgcn_sched_barrier(0);
    load_b(b1, s1);
    load_a(a0, s1, 0);
    __builtin_amdgcn_sched_barrier(0);
    mma(a1, b0, 1);
    __builtin_amdgcn_sched_barrier(0);
    load_a(a1, s1, 1);
    __builtin_amdgcn_sched_barrier(0);
    mma(a0, b1, 0);
    __builtin_amdgcn_sched_barrier(0);
    mma(a1, b1, 1);
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __syncthreads();
  }
  if (kt < KT) {   // odd number of K steps: the last one sits alone in its buffer's first stage
    const char* s0 = lds + (((kt >> 1) & 1) * 2) * kStageBytes;
    AFr a0, a1;
    BFr b0;
    load_b(b0, s0);
    load_a(a0, s0, 0);
    load_a(a1, s0, 1);
    mma(a0, b0, 0);
    mma(a1, b0, 1);
  }

  const float out_scale = A.ts[0] * B.ts[0];   // both are 1 for MXFP4 (no tensor-level scale)
  const int Mt = static_cast<int>(A.outer - m0 < TM ? A.outer - m0 : TM);
  const int Nt = static_cast<int>(B.outer - n0 < TN ? B.outer - n0 : TN);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int m = wm * 128 + i * 16 + l16;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = wn * 64 + j * 16 + kb * 4;
      if (m < Mt && n < Nt) {  // N is a multiple of 32, so the 4 columns are in or out together
        float4v v = acc[i][j] * out_scale;
        if (kBf16Out) {
          uint16_t* d = static_cast<uint16_t*>(Dv) + (m0 + m) * ldd + n0 + n;
          uint2 o;
          o.x = f32_to_bf16(v[0]) | (f32_to_bf16(v[1]) << 16);
          o.y = f32_to_bf16(v[2]) | (f32_to_bf16(v[3]) << 16);
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

hipError_t launch_gemm_mx(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = static_cast<int>((g.a.outer + TM - 1) / TM), tiles_n = static_cast<int>((g.b.outer + TN - 1) / TN);
  const dim3 grid(static_cast<unsigned>(tiles_m) * static_cast<unsigned>(tiles_n));
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mx_kernel<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 4 * kStageBytes);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mx_kernel<false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 4 * kStageBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (g.out_bf16)
    hipLaunchKernelGGL(gemm_mx_kernel<true>, grid, dim3(kThreads), 4 * kStageBytes, s, g.a, g.b, g.K, g.d, g.ldd,
                       g.accumulate, tiles_m, tiles_n);
  else
    hipLaunchKernelGGL(gemm_mx_kernel<false>, grid, dim3(kThreads), 4 * kStageBytes, s, g.a, g.b, g.K, g.d, g.ldd,
                       g.accumulate, tiles_m, tiles_n);
  return hipGetLastError();
}

}  // namespace nvfp4
