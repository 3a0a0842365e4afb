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
// 256 x 256 outputs per workgroup, K step 128 (one instruction deep), 256 threads = 4 wavefronts
// (2 x 2), one per SIMD, of 128 x 128 outputs each: 8 x 8 instructions per K step, 256 accumulator
// registers in the accumulation half of the register file.  LDS holds two buffers of two K steps,
// a step being (A codes, B codes, A scales, B scales) = 34 KiB, filled by direct global->LDS
// loads: a code row of a step is 64 bytes, so 16 consecutive tile rows are 1 KiB of LDS and a
// fragment read (16 rows x 4 blocks x 16 bytes) is one contiguous KiB.
//
// With one wavefront per SIMD nothing else can fill the matrix pipe while this one waits, so the
// loop is software-pipelined across its barrier and its instruction order is fixed by hand (inline
// assembly; the compiler would regroup it).  One iteration = the two K steps of a buffer:
//   block 1   64 MFMAs on the first step; behind them the 24 fragment reads of the second
//   wait      own reads back, own global->LDS loads (issued one iteration ago) landed; barrier:
//             every wavefront holds all it needs of this buffer, and the other buffer is complete
//   block 2   64 MFMAs on the second step; behind them the reads for the first step of the
//             other buffer and the 20 loads that refill this one with the steps after that
#include <type_traits>

#include "nvfp4_internal.h"
#include "nvfp4_device.h"
#include "gemm_epilogue.h"

namespace nvfp4 {

namespace {

constexpr int TM = 256, TN = 256, TK = 128;
constexpr int kThreads = 256;
constexpr int kCodeRowBytes = TK / 2;                 // 64
constexpr int kCodeBytes = TM * kCodeRowBytes;        // 16 KiB per operand
constexpr int kScaleBytes = TM * (TK / 32);           // 1 KiB per operand
constexpr int kStepBytes = 2 * kCodeBytes + 2 * kScaleBytes;   // 34 KiB
constexpr int kLdsBytes = 4 * kStepBytes;

typedef int int4v __attribute__((ext_vector_type(4)));

template <int kBegin, int kEnd, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (kBegin < kEnd) {
    f(std::integral_constant<int, kBegin>{});
    static_for<kBegin + 1, kEnd>(f);
  }
}

// 64 lanes x 16 (or 4) bytes from global memory (wave-uniform base + per-lane 32-bit offset) straight
// into consecutive LDS at the wave-uniform LDS address lds_dst (M0 carries it).  Asynchronous (vmcnt).
__device__ __forceinline__ void load16_to_lds(uint32_t lane_offset, const uint8_t* base, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_dst), "v"(lane_offset), "s"(base)
               : "memory", "m0");
}
__device__ __forceinline__ void load4_to_lds(uint32_t lane_offset, const uint8_t* base, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_dst), "v"(lane_offset), "s"(base)
               : "memory", "m0");
}

// LDS reads; asynchronous, the caller waits (lgkmcnt) before the values are used.
template <int kOff>
__device__ __forceinline__ void lds_read16(int4v& dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(kOff));
}
typedef int int2v __attribute__((ext_vector_type(2)));
// two dwords, kOff0 and kOff1 dwords past addr
template <int kOff0, int kOff1>
__device__ __forceinline__ void lds_read_2x4(int2v& dst, uint32_t addr) {
  asm volatile("ds_read2_b32 %0, %1 offset0:%2 offset1:%3" : "=&v"(dst) : "v"(addr), "n"(kOff0), "n"(kOff1));
}
// byte k of the result = byte sel[k] of the eight bytes {hi, lo}; in assembly so that it stays behind the
// wait for the LDS reads that produce its inputs (the compiler does not know those are asynchronous)
__device__ __forceinline__ int perm_bytes(int hi, int lo, int sel) {
  int d;
  asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(d) : "v"(hi), "v"(lo), "v"(sel));
  return d;
}

// Fragments of one K step for a 128 x 128 wave tile: per 16-row block the lane's 32 codes (the
// instruction's FP4 operand is four dwords) and its block's scale byte.  Single-byte LDS reads are slow
// (measured: 16 of them per K step cost more than the 64 MFMAs), so the scales are read as the row's whole
// dword (the step's four blocks) and the lane's own byte of four rows is gathered into one register (pa, pb);
// the instruction then picks the row's byte with its op_sel field.
constexpr int kFragReads = 24;
struct Frags {
  int4v a[8], b[8];
  int pa[2], pb[2];     // byte t of pa[h] = this lane's scale of block 4h + t
};
// Raw scale dwords of 16-row blocks (2t, 2t + 1) between their read and the gather; one set serves both
// fragment sets, whose reads never overlap (each set is gathered before the other's reads start).
struct RawScales {
  int2v a[4], b[4];
};

// Read number q of the 24 of a fragment set: 0..7 A codes, 8..15 B codes, 16..19 A scales, 20..23 B scales
// (16-row blocks are 1 KiB of codes and 64 bytes = 16 dwords of scales apart).
template <int q>
__device__ __forceinline__ void read_frag(Frags& f, RawScales& r, uint32_t a_codes, uint32_t b_codes, uint32_t a_scales,
                                          uint32_t b_scales) {
  if constexpr (q < 8) lds_read16<q * 16 * kCodeRowBytes>(f.a[q], a_codes);
  else if constexpr (q < 16) lds_read16<(q - 8) * 16 * kCodeRowBytes>(f.b[q - 8], b_codes);
  else if constexpr (q < 20) lds_read_2x4<(q - 16) * 32, (q - 16) * 32 + 16>(r.a[q - 16], a_scales);
  else lds_read_2x4<(q - 20) * 32, (q - 20) * 32 + 16>(r.b[q - 20], b_scales);
}

// After the reads are back: gather the lane's byte (sel01 = kb | (4 + kb) << 8 picks byte kb of two dwords).
__device__ __forceinline__ void pack_scales(Frags& f, const RawScales& r, int sel01) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int a01 = perm_bytes(r.a[2 * h][1], r.a[2 * h][0], sel01), a23 = perm_bytes(r.a[2 * h + 1][1], r.a[2 * h + 1][0], sel01);
    f.pa[h] = perm_bytes(a23, a01, 0x05040100);
    const int b01 = perm_bytes(r.b[2 * h][1], r.b[2 * h][0], sel01), b23 = perm_bytes(r.b[2 * h + 1][1], r.b[2 * h + 1][0], sel01);
    f.pb[h] = perm_bytes(b23, b01, 0x05040100);
  }
}

// The instruction's first operand supplies the rows of its result: passing B first leaves a lane with 4
// consecutive n of one m, which makes the output stores 64/128-bit.  cbsz / blgp = 4: both operands FP4;
// scale byte kSelB of sb and kSelA of sa (op_sel = the low bit, op_sel_hi = the high bit of the byte number).
// The accumulator is pinned to the accumulation registers.
template <int kSelB, int kSelA>
__device__ __forceinline__ void mfma(float4v& acc, const int4v& b, const int4v& a, int sb, int sa) {
  asm volatile("v_mfma_scale_f32_16x16x128_f8f6f4 %0, %1, %2, %0, %3, %4 op_sel:[%5,%6,0] op_sel_hi:[%7,%8,0] cbsz:4 blgp:4"
               : "+a"(acc)
               : "v"(b), "v"(a), "v"(sb), "v"(sa), "n"(kSelB & 1), "n"(kSelA & 1), "n"(kSelB >> 1), "n"(kSelA >> 1));
}

template <bool kBf16Out>
__global__ __launch_bounds__(kThreads) void gemm_mx_kernel_any_k(Operand A, Operand B, int64_t K, void* __restrict__ Dv,
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
  const int wm = wave >> 1, wn = wave & 1, l16 = lane & 15, kb = lane >> 4;
  const int arow = wm * 128 + l16, brow = wn * 128 + l16;
  const int64_t code_ld = K / 2, scale_ld = K / 32;

  // Direct-load sources = wave-uniform 64-bit base + per-lane 32-bit offset.  Codes: an instruction fills 16 tile
  // rows (lane -> row lane / 4, 16-byte piece lane % 4), so one per-lane offset serves every instruction and both
  // operands (a 16-row block is at most 16 * K / 2 bytes: K < 2^24, checked on the host); every wavefront loads 64
  // rows of A and of B.  A 16-row block past the end of an operand is replaced by the operand's last block (rows
  // come in multiples of 32, so a block is in or out as a whole); it only feeds outputs that are never stored.
  // Scales: an instruction fills 64 tile rows x 4 bytes, rows clamped per lane; every wavefront loads its 64 rows.
  const uint32_t off_codes = static_cast<uint32_t>(lane >> 2) * static_cast<uint32_t>(code_ld) + (lane & 3) * 16;
  const uint32_t off_sa = static_cast<uint32_t>(min<int64_t>(wave * 64 + lane, A.outer - 1 - m0)) * static_cast<uint32_t>(scale_ld);
  const uint32_t off_sb = static_cast<uint32_t>(min<int64_t>(wave * 64 + lane, B.outer - 1 - n0)) * static_cast<uint32_t>(scale_ld);
  const uint8_t* tile_sa = A.scales + m0 * scale_ld;
  const uint8_t* tile_sb = B.scales + n0 * scale_ld;
  const uint8_t* blk_a[4];
  const uint8_t* blk_b[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int64_t r = (wave * 4 + q) * 16;
    blk_a[q] = A.codes + (m0 + min<int64_t>(r, A.outer - 16 - m0)) * code_ld;
    blk_b[q] = B.codes + (n0 + min<int64_t>(r, B.outer - 16 - n0)) * code_ld;
  }
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));
  // load number q (0..9) of K step kt into step slot `slot` (0..3): 0..3 A codes, 4..7 B codes, 8 A scales, 9 B scales
  auto issue_one = [&](int q, int kt, int slot) {
    const uint32_t base = lds0 + slot * kStepBytes;
    if (q < 4)
      load16_to_lds(off_codes, blk_a[q & 3] + static_cast<int64_t>(kt) * kCodeRowBytes, base + (wave * 4 + q) * 1024);
    else if (q < 8)
      load16_to_lds(off_codes, blk_b[q & 3] + static_cast<int64_t>(kt) * kCodeRowBytes, base + kCodeBytes + (wave * 4 + (q & 3)) * 1024);
    else if (q == 8)
      load4_to_lds(off_sa, tile_sa + static_cast<int64_t>(kt) * 4, base + 2 * kCodeBytes + wave * 256);
    else
      load4_to_lds(off_sb, tile_sb + static_cast<int64_t>(kt) * 4, base + 2 * kCodeBytes + kScaleBytes + wave * 256);
  };
  // fragment addresses in step slot 0
  const uint32_t a_codes = lds0 + arow * kCodeRowBytes + kb * 16, b_codes = lds0 + kCodeBytes + brow * kCodeRowBytes + kb * 16;
  const uint32_t a_scales = lds0 + 2 * kCodeBytes + arow * 4, b_scales = lds0 + 2 * kCodeBytes + kScaleBytes + brow * 4;
  const int sel01 = kb | ((4 + kb) << 8);

  float4v acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

  const int KT = static_cast<int>(K / TK);
  // K steps 0..3 into step slots 0..3.  Steps past the end are clamped to the last one: they land in slots nobody
  // multiplies any more, and no branch is needed.
  static_for<0, 40>([&](auto ic) {
    constexpr int n = decltype(ic)::value;
    issue_one(n % 10, min(n / 10, KT - 1), n / 10);
  });
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  Frags f0, f1;
  RawScales raw;
  static_for<0, kFragReads>([&](auto q) { read_frag<decltype(q)::value>(f0, raw, a_codes, b_codes, a_scales, b_scales); });
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  pack_scales(f0, raw, sel01);

  for (int kt = 0; kt < KT; kt += 2) {
    const uint32_t cur = ((kt >> 1) & 1) * (2 * kStepBytes), nxt = cur ^ (2 * kStepBytes);
    const uint32_t second = cur + kStepBytes;
    static_for<0, 64>([&](auto ic) {
      constexpr int n = decltype(ic)::value;
      mfma<(n & 3), ((n >> 3) & 3)>(acc[n >> 3][n & 7], f0.b[n & 7], f0.a[n >> 3], f0.pb[(n & 7) >> 2], f0.pa[n >> 5]);
      if constexpr ((n & 1) == 1 && (n >> 1) < kFragReads)
        read_frag<(n >> 1)>(f1, raw, a_codes + second, b_codes + second, a_scales + second, b_scales + second);
    });
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    pack_scales(f1, raw, sel01);
    if (kt + 1 < KT) {   // an odd number of K steps leaves the last buffer's second step empty
      const int slot = ((kt >> 1) & 1) * 2;
      const int kt4 = min(kt + 4, KT - 1), kt5 = min(kt + 5, KT - 1);
      static_for<0, 64>([&](auto ic) {
        constexpr int n = decltype(ic)::value;
        mfma<(n & 3), ((n >> 3) & 3)>(acc[n >> 3][n & 7], f1.b[n & 7], f1.a[n >> 3], f1.pb[(n & 7) >> 2], f1.pa[n >> 5]);
        if constexpr ((n & 1) == 0 && (n >> 1) < kFragReads)
          read_frag<(n >> 1)>(f0, raw, a_codes + nxt, b_codes + nxt, a_scales + nxt, b_scales + nxt);
        if constexpr ((n & 1) == 1 && n < 40)
          issue_one((n >> 1) % 10, (n >> 1) < 10 ? kt4 : kt5, slot + ((n >> 1) < 10 ? 0 : 1));
      });
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      pack_scales(f0, raw, sel01);
    }
  }
  // The trailing global->LDS loads must have landed before the wavefront ends; the MFMA results must have left
  // the pipe before ordinary instructions read the accumulators (the compiler cannot see into the assembly
  // statements to insert these wait states itself).
  asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");

  const TensorScales out_scale{A.ts, B.ts, false, false};    // both are 1 for MXFP4 (no tensor-level scale)
  const int Mt = static_cast<int>(A.outer - m0 < TM ? A.outer - m0 : TM);
  const int Nt = static_cast<int>(B.outer - n0 < TN ? B.outer - n0 : TN);
  store_wave_block<kBf16Out>(acc, out_scale, Dv, ldd, accumulate, m0 + wm * 128, n0 + wn * 128, Mt - wm * 128, Nt - wn * 128,
                             lane);
}

// ---------------------------------------------------------------- K a multiple of 512
// The kernel above asks the memory system for many small pieces: per K step a 64-byte piece of every code row
// and a 4-byte piece of every scale row, each its own cache-line request (measured: about one request per
// clock and CU, which is what bounds it).  When K is a multiple of 512 the same loop runs on fuller lines:
//   codes   a stage is two K steps = 128 bytes of each row, 8 rows per load instruction, stored with the XOR
//           swizzle chunk c of row r -> position c ^ ((r >> 1) & 7) so that fragment reads stay conflict-free;
//           the two steps of an iteration are the two 64-byte halves of a stage
//   scales  16 bytes of each scale row = four K steps = two iterations per load instruction, in a ring of
//           two 8 KiB slots; a lane reads its row's dword of the step and gathers bytes as before
// a third of the line requests for the same bytes.  The pipeline is the one described at the top.
constexpr int kWideRowBytes = 128;
constexpr int kWideOperandBytes = TM * kWideRowBytes;       // 32 KiB
constexpr int kWideStageBytes = 2 * kWideOperandBytes;      // 64 KiB
constexpr int kWideScaleOperandBytes = TM * 16;             // 4 KiB: 256 rows x 4 steps x 4 blocks
constexpr int kWideScaleSlotBytes = 2 * kWideScaleOperandBytes;
constexpr int kWideLdsBytes = 2 * kWideStageBytes + 2 * kWideScaleSlotBytes;   // 144 KiB

__device__ __forceinline__ int swz128(int row, int chunk) { return row * kWideRowBytes + ((chunk ^ ((row >> 1) & 7)) << 4); }

// two dwords, kOff0 and kOff1 times 256 bytes past addr
template <int kOff0, int kOff1>
__device__ __forceinline__ void lds_read_2x4_st64(int2v& dst, uint32_t addr) {
  asm volatile("ds_read2st64_b32 %0, %1 offset0:%2 offset1:%3" : "=&v"(dst) : "v"(addr), "n"(kOff0), "n"(kOff1));
}

// Read number q of the 24 of a fragment set: 0..7 A codes, 8..15 B codes (16-row blocks are 2 KiB apart), 16..19 A
// scales, 20..23 B scales (16-row blocks are 256 bytes apart).
template <int q>
__device__ __forceinline__ void read_frag_wide(Frags& f, RawScales& r, uint32_t a_codes, uint32_t b_codes, uint32_t a_scales,
                                               uint32_t b_scales) {
  if constexpr (q < 8) lds_read16<q * 16 * kWideRowBytes>(f.a[q], a_codes);
  else if constexpr (q < 16) lds_read16<(q - 8) * 16 * kWideRowBytes>(f.b[q - 8], b_codes);
  else if constexpr (q < 20) lds_read_2x4_st64<(q - 16) * 2, (q - 16) * 2 + 1>(r.a[q - 16], a_scales);
  else lds_read_2x4_st64<(q - 20) * 2, (q - 20) * 2 + 1>(r.b[q - 20], b_scales);
}

// The first instruction on an accumulator in a tile: C = 0, so the 256 accumulation registers are never cleared.
template <int kSelB, int kSelA>
__device__ __forceinline__ void mfma_first(float4v& acc, const int4v& b, const int4v& a, int sb, int sa) {
  asm volatile("v_mfma_scale_f32_16x16x128_f8f6f4 %0, %1, %2, 0, %3, %4 op_sel:[%5,%6,0] op_sel_hi:[%7,%8,0] cbsz:4 blgp:4"
               : "=a"(acc)
               : "v"(b), "v"(a), "v"(sb), "v"(sa), "n"(kSelB & 1), "n"(kSelA & 1), "n"(kSelB >> 1), "n"(kSelA >> 1));
}

// A wavefront's output stage issues 32 (bf16) or 64 (FP32) stores for a full tile; three quarters of them may still be
// outstanding when the loads issued before it are needed (memory operations complete in issue order).
template <bool kBf16Out>
constexpr int kTileStoresMx = kBf16Out ? 24 : 48;

// With more tiles than CUs the host launches one workgroup per CU, which takes tiles blockIdx.x, blockIdx.x +
// gridDim.x, ... and runs them as ONE stream of stages, as the FP16 kernel of the NVFP4 route does: the loads issued
// during a tile's last two stages fetch the next tile's first two (and its first scale chunk), so the pipeline
// neither drains nor refills at a tile boundary.  K is a multiple of 512, so every tile is an even number of stages
// and a whole number of scale chunks: the stage buffers and the scale ring simply keep turning (`gst` below counts
// stages over all tiles).  The output stage's stores are not waited for.
template <bool kBf16Out>
__global__ __launch_bounds__(kThreads) void gemm_mx_kernel_k512(Operand A, Operand B, int64_t K, void* __restrict__ Dv,
                                                                int64_t ldd, bool accumulate, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) char lds[];

  const int num_tiles = tiles_m * tiles_n;
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) >> 6);
  const int64_t code_ld = K / 2, scale_ld = K / 32;
  // Work item -> tile: consecutive workgroup ids go to different XCDs (round robin over 8, one L2 each); every XCD
  // gets a contiguous range of tiles, walked in bands of 8 tile rows.
  auto locate = [&](int item, int& tm, int& tn) {
    if ((num_tiles & 7) == 0) item = (item & 7) * (num_tiles >> 3) + (item >> 3);
    tile_coordinates(item, tiles_m, tiles_n, tm, tn);
  };

  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));
  const uint32_t scales0 = lds0 + 2 * kWideStageBytes;
  // What depends on the lane is worked out once per tile, from a lane number asked for on the spot (values kept from
  // before the first tile would have to live through every output stage and end up in scratch memory).
  // Code loads: instruction q (0..7) of wavefront w fills tile rows w * 64 + 8 q .. + 7 (lane -> row lane / 8,
  // position lane % 8, i.e. chunk (lane % 8) ^ ((row >> 1) & 7); 8 q leaves that term alone for even q and flips
  // its bit 2 for odd q).  Scale loads: one instruction = 64 tile rows x 16 bytes (four K steps).
  uint32_t lane_even = 0, lane_odd = 0, lane_srow = 0;
  uint32_t a_lo = 0, a_hi = 0, b_lo = 0, b_hi = 0, a_scales = 0, b_scales = 0;   // fragment addresses: stage buffer 0 / scale slot 0, step 0
  int sel01 = 0;
  auto lane_setup = [&]() {
    const int lane = lane_id();
    const int r0 = wave * 64 + (lane >> 3);
    const uint32_t c0 = static_cast<uint32_t>((lane & 7) ^ ((r0 >> 1) & 7)) * 16u;
    lane_even = static_cast<uint32_t>(lane >> 3) * static_cast<uint32_t>(code_ld) + c0;
    lane_odd = static_cast<uint32_t>(lane >> 3) * static_cast<uint32_t>(code_ld) + (c0 ^ 64u);
    lane_srow = static_cast<uint32_t>(wave * 64 + lane);
    const int l16 = lane & 15, kb = lane >> 4;
    const int arow = (wave >> 1) * 128 + l16, brow = (wave & 1) * 128 + l16;
    a_lo = lds0 + swz128(arow, kb);
    a_hi = lds0 + swz128(arow, 4 + kb);
    b_lo = lds0 + kWideOperandBytes + swz128(brow, kb);
    b_hi = lds0 + kWideOperandBytes + swz128(brow, 4 + kb);
    a_scales = scales0 + arow * 16;
    b_scales = scales0 + kWideScaleOperandBytes + brow * 16;
    sel01 = kb | ((4 + kb) << 8);
  };
  lane_setup();
  // Load addresses: a wave-uniform 64-bit base per operand (codes, scales), which holds the tile and the stage /
  // scale chunk being fetched, plus per-lane 32-bit offsets, which hold the row and the chunk and do not change
  // within a tile (256 rows of K / 2 bytes: K < 2^24, checked on the host): moving the loads on is scalar work.  An 8-row block past the end of an operand is replaced by the operand's last block (rows come in
  // multiples of 32); it only feeds outputs that are never stored.  Scale rows are clamped per lane.
  const uint8_t* base_a = nullptr;
  const uint8_t* base_b = nullptr;
  const uint8_t* base_sa = nullptr;
  const uint8_t* base_sb = nullptr;
  uint32_t voff[16];   // q 0..7 A, 8..15 B
  uint32_t vsa = 0, vsb = 0;
  // Point the loads at stage `stage` and scale chunk `chunk` of tile (tm, tn).
  auto aim = [&](int tm, int tn, int stage, int chunk) {
    const int64_t m_first = static_cast<int64_t>(tm) * TM, n_first = static_cast<int64_t>(tn) * TN;
    base_a = A.codes + m_first * code_ld + stage * kWideRowBytes;
    base_b = B.codes + n_first * code_ld + stage * kWideRowBytes;
    base_sa = A.scales + m_first * scale_ld + chunk * 16;
    base_sb = B.scales + n_first * scale_ld + chunk * 16;
    const uint32_t last_a = static_cast<uint32_t>(A.outer - 8 - m_first), last_b = static_cast<uint32_t>(B.outer - 8 - n_first);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const uint32_t r = static_cast<uint32_t>(wave * 64 + q * 8);
      voff[q] = ((q & 1) ? lane_odd : lane_even) + min(r, last_a) * static_cast<uint32_t>(code_ld);
      voff[8 + q] = ((q & 1) ? lane_odd : lane_even) + min(r, last_b) * static_cast<uint32_t>(code_ld);
    }
    vsa = min(lane_srow, last_a + 7) * static_cast<uint32_t>(scale_ld);
    vsb = min(lane_srow, last_b + 7) * static_cast<uint32_t>(scale_ld);
  };
  // load number q (0..15) of a stage into stage buffer `buf`: 0..7 A, 8..15 B
  auto issue_codes = [&](auto qc, int buf) {
    constexpr int q = decltype(qc)::value;
    const uint32_t dst = lds0 + buf * kWideStageBytes + (q < 8 ? 0 : kWideOperandBytes) + wave * 8192 + (q & 7) * 1024;
    load16_to_lds(voff[q], q < 8 ? base_a : base_b, dst);
  };
  // the two loads of a scale chunk (four K steps) into ring slot `slot`
  auto issue_scales = [&](int slot) {
    const uint32_t dst = scales0 + slot * kWideScaleSlotBytes + wave * 1024;
    load16_to_lds(vsa, base_sa, dst);
    load16_to_lds(vsb, base_sb, dst + kWideScaleOperandBytes);
  };

  const int stages = static_cast<int>(K / 256), chunks = static_cast<int>(K / 512);   // stages = 2 chunks >= 2
  int item = blockIdx.x;   // < num_tiles: the host launches at most that many workgroups
  int tm = 0, tn = 0;
  locate(item, tm, tn);
  aim(tm, tn, 0, 0);
  static_for<0, 16>([&](auto q) { issue_codes(q, 0); });
  base_a += kWideRowBytes;
  base_b += kWideRowBytes;
  static_for<0, 16>([&](auto q) { issue_codes(q, 1); });
  issue_scales(0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();

  Frags f0, f1;
  RawScales raw;
  float4v acc[8][8];
  uint32_t gst = 0;             // stages done so far, over all tiles (even at every tile's start)
  bool stores_behind = false;   // the previous tile's stores were issued after the loads now in flight
  for (;;) {
    // The tile's first fragments.  (After a tile of the same stream its last stage has read them already; they are
    // read again so that the output stage had their registers to work with.)
    {
      const uint32_t cur = (gst & 1) * kWideStageBytes, sc = ((gst >> 1) & 1) * kWideScaleSlotBytes;
      static_for<0, kFragReads>([&](auto q) { read_frag_wide<decltype(q)::value>(f0, raw, a_lo + cur, b_lo + cur, a_scales + sc, b_scales + sc); });
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      pack_scales(f0, raw, sel01);
    }
    const int next_item = item + static_cast<int>(gridDim.x);
    const bool has_next = next_item < num_tiles;
    int next_tm = 0, next_tn = 0;
    if (has_next) locate(next_item, next_tm, next_tn);

    // One stage = two K steps; kFirst: the tile's first.  The loads run two stages ahead of the MFMAs, the scale
    // loads (every other stage) one chunk ahead of the stage that reads it.
    auto stage_step = [&](auto first_tag, int st) {
      constexpr bool kFirst = decltype(first_tag)::value;
      const uint32_t cur = (gst & 1) * kWideStageBytes, nxt = cur ^ kWideStageBytes;
      // scale addresses: this stage's second step; the next stage's first step (ring slot of its chunk)
      const uint32_t sc1 = ((gst >> 1) & 1) * kWideScaleSlotBytes + (gst & 1) * 8 + 4;
      const uint32_t sc2 = (((gst + 1) >> 1) & 1) * kWideScaleSlotBytes + ((gst + 1) & 1) * 8;
      // Where the loads go next: on within the tile, or to the next tile's first stage and chunk, or, with nothing
      // to follow, nowhere (the last stage and chunk are fetched again into buffers nobody reads any more).
      uint32_t code_advance = kWideRowBytes;
      if ((st & 1) == 0 && (st >> 1) + 1 < chunks) {
        base_sa += 16;
        base_sb += 16;
      }
      if (st + 2 == stages) {
        code_advance = 0;
        if (has_next) aim(next_tm, next_tn, 0, 0);
      } else if (st + 2 > stages && !has_next) {
        code_advance = 0;
      }
      static_for<0, 64>([&](auto ic) {
        constexpr int n = decltype(ic)::value;
        if constexpr (kFirst)
          mfma_first<(n & 3), ((n >> 3) & 3)>(acc[n >> 3][n & 7], f0.b[n & 7], f0.a[n >> 3], f0.pb[(n & 7) >> 2], f0.pa[n >> 5]);
        else
          mfma<(n & 3), ((n >> 3) & 3)>(acc[n >> 3][n & 7], f0.b[n & 7], f0.a[n >> 3], f0.pb[(n & 7) >> 2], f0.pa[n >> 5]);
        if constexpr ((n & 1) == 1 && (n >> 1) < kFragReads)
          read_frag_wide<(n >> 1)>(f1, raw, a_hi + cur, b_hi + cur, a_scales + sc1, b_scales + sc1);
        if constexpr (n == 2) {
          base_a += code_advance;
          base_b += code_advance;
        }
      });
      if (kFirst && stores_behind) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(kTileStoresMx<kBf16Out>) : "memory");
      else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      pack_scales(f1, raw, sel01);
      static_for<0, 64>([&](auto ic) {
        constexpr int n = decltype(ic)::value;
        mfma<(n & 3), ((n >> 3) & 3)>(acc[n >> 3][n & 7], f1.b[n & 7], f1.a[n >> 3], f1.pb[(n & 7) >> 2], f1.pa[n >> 5]);
        if constexpr ((n & 1) == 0 && (n >> 1) < kFragReads)
          read_frag_wide<(n >> 1)>(f0, raw, a_lo + nxt, b_lo + nxt, a_scales + sc2, b_scales + sc2);
        if constexpr ((n & 3) == 3) issue_codes(std::integral_constant<int, (n >> 2)>{}, static_cast<int>(gst & 1));
      });
      // even stages also fetch the scales of the chunk after the next stage's, into the slot its predecessor left
      // at this stage's barrier
      if ((gst & 1) == 0) issue_scales(static_cast<int>(((gst >> 1) + 1) & 1));
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      pack_scales(f0, raw, sel01);
      ++gst;
    };
    stage_step(std::true_type{}, 0);
    for (int st = 1; st < stages; ++st) stage_step(std::false_type{}, st);

    // Everything below is computed here, per tile (see lane_setup).
    int wm = wave >> 1, wn = wave & 1;
    asm volatile("" : "+s"(wm), "+s"(wn));
    const int lane = lane_id();
    const TensorScales out_scale{A.ts, B.ts, false, false};    // both are 1 for MXFP4 (no tensor-level scale)
    const int64_t m0 = static_cast<int64_t>(tm) * TM, n0 = static_cast<int64_t>(tn) * TN;
    const int Mt = static_cast<int>(A.outer - m0 < TM ? A.outer - m0 : TM);
    const int Nt = static_cast<int>(B.outer - n0 < TN ? B.outer - n0 : TN);
    // The MFMA results must have left the pipe before ordinary instructions read the accumulators (the compiler
    // cannot see into the assembly statements to insert these wait states itself).  With nothing to follow, the
    // trailing global->LDS loads must have landed before the wavefront ends.
    if (has_next) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    store_wave_block<kBf16Out>(acc, out_scale, Dv, ldd, accumulate, m0 + wm * 128, n0 + wn * 128, Mt - wm * 128, Nt - wn * 128,
                               lane);
    if (!has_next) break;
    stores_behind = Mt == TM && Nt == TN;   // every lane stored every block: the count is known
    item = next_item;
    tm = next_tm;
    tn = next_tn;
    lane_setup();
    aim(tm, tn, 1, 0);   // where the loads stand: the tile's second stage and first scale chunk are the last fetched
  }
}

}  // namespace

template <class Kernel>
static hipError_t launch_mx(Kernel kernel, PerDeviceOnce& once, int lds_bytes, const GemmArgs& g, dim3 grid, int tiles_m, int tiles_n,
                            hipStream_t s) {
  const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kernel), lds_bytes, once);   // more dynamic LDS than the default limit
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds_bytes, s, g.a, g.b, g.K, g.d, g.ldd, g.accumulate, tiles_m, tiles_n);
  return hipGetLastError();
}

hipError_t launch_gemm_mx(const GemmArgs& g, hipStream_t s) {
  if (g.K >= (int64_t{1} << 24)) return hipErrorInvalidValue;   // the kernels' 32-bit byte offsets inside a block of rows
  const int tiles_m = static_cast<int>((g.a.outer + TM - 1) / TM), tiles_n = static_cast<int>((g.b.outer + TN - 1) / TN);
  const unsigned tiles = static_cast<unsigned>(tiles_m) * static_cast<unsigned>(tiles_n);
  const dim3 grid(tiles);
  const dim3 grid_cus(tiles < 256u ? tiles : 256u);   // the k512 kernel: one workgroup per CU, each running its tiles as one stream
  // 16-byte pieces of scale rows need K / 32 to be a multiple of 16 and the scale arrays 16-byte aligned
  const bool wide = g.K % 512 == 0 && reinterpret_cast<uintptr_t>(g.a.scales) % 16 == 0 && reinterpret_cast<uintptr_t>(g.b.scales) % 16 == 0;
  static PerDeviceOnce set[4];
  if (wide) {
    if (g.out_bf16) return launch_mx(gemm_mx_kernel_k512<true>, set[0], kWideLdsBytes, g, grid_cus, tiles_m, tiles_n, s);
    return launch_mx(gemm_mx_kernel_k512<false>, set[1], kWideLdsBytes, g, grid_cus, tiles_m, tiles_n, s);
  }
  if (g.out_bf16) return launch_mx(gemm_mx_kernel_any_k<true>, set[2], kLdsBytes, g, grid, tiles_m, tiles_n, s);
  return launch_mx(gemm_mx_kernel_any_k<false>, set[3], kLdsBytes, g, grid, tiles_m, tiles_n, s);
}

}  // namespace nvfp4
