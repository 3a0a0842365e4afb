// Two-pass form of the block-scaled GEMM (App. B.3 Eq. 5) for gfx950, used when
// the caller lends a workspace:
//   pass 1  decode both NVFP4 operands to FP16, value * block_scale (exact: the
//           product has at most 6 significant bits), K-contiguous, into the
//           workspace;
//   pass 2  a plain FP16 x FP16 -> FP32 MFMA GEMM whose main loop has no VALU
//           work at all: tiles go from global memory straight into LDS
//           (global_load_lds_dwordx4), fragments come from LDS, 16x16x32 MFMAs
//           (measured under the chip's power limit: a register-only loop of
//           v_mfma_f32_16x16x32_f16 sustains 12-20 % more flop/s than one of
//           v_mfma_f32_32x32x16_f16 on the same operand values).
// Why: decoding inside the GEMM loop costs about one VALU instruction per
// element, and VALU instructions co-issued with MFMAs take matrix-pipe time
// (measured: the fused kernel runs at 1.0-1.07 PFLOP/s, this pair at about
// 1.39 PFLOP/s in the GEMM proper, the decode pass adding 5-8 % of its time).
// The results are identical to the fused kernel's up to FP32 summation order.
#include <type_traits>

#include "nvfp4_internal.h"
#include "nvfp4_device.h"
#include "gemm_epilogue.h"

namespace nvfp4 {

namespace {

// ---------------------------------------------------------------- pass 1: decode
template <int kByte>
__device__ __forceinline__ half2v dec_pair(uint32_t codes, half2v scale) {
  return __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 1.0f, kByte) * scale;
}

__device__ __forceinline__ uint4 dec8(uint32_t codes, half2v scale) {
  union {
    half2v h[4];
    uint4 u;
  } o;
  o.h[0] = dec_pair<0>(codes, scale);
  o.h[1] = dec_pair<1>(codes, scale);
  o.h[2] = dec_pair<2>(codes, scale);
  o.h[3] = dec_pair<3>(codes, scale);
  return o.u;
}

__device__ __forceinline__ half2v scale_h2(uint32_t e4m3_byte) {
  const _Float16 s = static_cast<_Float16>(e4m3_decode(e4m3_byte));
  half2v r;
  r.x = s;
  r.y = s;
  return r;
}

// A thread decodes kDecodeUnroll x 8 elements (a dword of codes -> 16 bytes of FP16 each), the pieces 256 dwords
// apart: consecutive lanes read consecutive dwords and write consecutive 16-byte pieces, so every load and store
// instruction of a wavefront covers one contiguous span, and a thread has all its loads in flight before its first
// store.  Both operands are decoded by one launch.
constexpr int kDecodeUnroll = 4;
__global__ __launch_bounds__(256) void decode_f16_kernel(const uint8_t* __restrict__ a_codes,
                                                         const uint8_t* __restrict__ a_scales, int64_t a_n8,
                                                         _Float16* __restrict__ a_out,
                                                         const uint8_t* __restrict__ b_codes,
                                                         const uint8_t* __restrict__ b_scales, int64_t b_n8,
                                                         _Float16* __restrict__ b_out,
                                                         unsigned int* __restrict__ tickets) {
  // The split-K tickets of the GEMM launches that follow start at zero (256 of them at most).
  if (blockIdx.x == 0 && tickets) tickets[threadIdx.x] = 0u;
  const int64_t base = static_cast<int64_t>(blockIdx.x) * (256 * kDecodeUnroll) + threadIdx.x;
  uint32_t c[kDecodeUnroll];
  uint32_t sc[kDecodeUnroll];
  uint4* dst[kDecodeUnroll];
#pragma unroll
  for (int u = 0; u < kDecodeUnroll; ++u) {
    int64_t i = base + u * 256;
    const bool in_a = i < a_n8;
    if (!in_a) i -= a_n8;
    dst[u] = nullptr;
    c[u] = 0u;
    sc[u] = 0u;
    if (in_a || i < b_n8) {
      c[u] = reinterpret_cast<const uint32_t*>(in_a ? a_codes : b_codes)[i];
      sc[u] = (in_a ? a_scales : b_scales)[i >> 1];
      dst[u] = reinterpret_cast<uint4*>(in_a ? a_out : b_out) + i;
    }
  }
#pragma unroll
  for (int u = 0; u < kDecodeUnroll; ++u)
    if (dst[u]) *dst[u] = dec8(c[u], scale_h2(sc[u]));
}

// ---------------------------------------------------------------- pass 2: FP16 GEMM
// 256 x 256 outputs per workgroup, K step 64, 256 threads = 4 wavefronts (2 x 2), one per SIMD,
// each 128 x 128 outputs as 8 x 8 MFMA 16x16 blocks: 256 accumulator registers, which live in
// the accumulation half of the register file, and 16 fragment loads per 64 MFMAs (a 128 x 64
// wave tile needs 12 per 32).  LDS holds two stages of (A tile, B tile), 64 KiB each; a stage is
// filled by direct global->LDS loads: one instruction moves 64 lanes x 16 bytes into 1 KiB of
// consecutive LDS, i.e. 8 tile rows of 128 bytes, and lane l fetches the 16-byte chunk that
// belongs at chunk position l & 7 of row l >> 3 under the XOR swizzle
// (chunk c of row r lives at position c ^ ((r >> 1) & 7)).
//
// With one wavefront per SIMD nothing else can fill the matrix pipe while this one waits, so the
// loop is software-pipelined across its barrier and its instruction order is fixed by hand (inline
// assembly keeps the compiler from regrouping it; measured 1.18 against 1.06 PFLOP/s for the
// 8-wavefront form on the same operands, at a lower clock: the chip's power limit sets the speed,
// and this form moves a third less data from LDS per flop):
//   block 1   64 MFMAs on the first 32 k of the stage; after every fourth, one of the 16 fragment
//             loads for the second 32 k
//   wait      own fragment loads back, own global->LDS loads (issued one step ago) landed; barrier:
//             every wavefront holds all it needs of this stage, and the next stage is complete
//   block 2   64 MFMAs on the second 32 k; after every second, alternately one fragment load for
//             the first 32 k of the next stage and one global->LDS load of the stage after that,
//             into the buffer just freed
// so the barrier falls between two blocks of MFMAs that are already fed.
constexpr int TM = 256, TN = 256, TK = 64;
constexpr int kThreads = 256;
constexpr int kRowBytes = TK * 2;
constexpr int kOperandBytes = TM * kRowBytes;   // 32 KiB
constexpr int kStageBytes = 2 * kOperandBytes;  // 64 KiB
constexpr int kLdsBytes = 2 * kStageBytes;

__device__ __forceinline__ int swz(int row, int chunk) { return row * kRowBytes + ((chunk ^ ((row >> 1) & 7)) << 4); }

// Fragments of one 32-wide half of a K step for a 128 x 128 wave tile.  A 16x16x32 MFMA operand
// is 16 rows x 32 k: lane l holds the 8 consecutive k of 16-byte chunk (l >> 4) of row (l & 15).
struct Frags {
  half8v a[8], b[8];
};

template <int kBegin, int kEnd, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (kBegin < kEnd) {
    f(std::integral_constant<int, kBegin>{});
    static_for<kBegin + 1, kEnd>(f);
  }
}

// The MFMA's M index is the B row (n), its N index the A row (m): lane l ends up with the 4
// consecutive n = (l >> 4) * 4 .. + 3 of m = l & 15, which makes the output stores 64/128-bit.
// The accumulator is pinned to the accumulation registers ("a"): 256 of them leave the 256
// ordinary registers to fragments and addresses.
__device__ __forceinline__ void mfma(float4v& acc, const half8v& b, const half8v& a) {
  asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(b), "v"(a));
}

// 16 bytes of LDS at addr + kOff.  Asynchronous: the caller waits (lgkmcnt) before the value is used.
template <int kOff>
__device__ __forceinline__ void lds_read16(half8v& dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(kOff));
}

// Fragment q of a 16-fragment set: 0..7 = A rows i * 16, 8..15 = B rows j * 16 (2 KiB apart; the
// swizzle term does not change with multiples of 16 rows).
template <int q>
__device__ __forceinline__ void read_frag(Frags& f, uint32_t a_addr, uint32_t b_addr) {
  if constexpr (q < 8) lds_read16<q * 16 * kRowBytes>(f.a[q], a_addr);
  else lds_read16<(q - 8) * 16 * kRowBytes>(f.b[q - 8], b_addr);
}

// 64 lanes x 16 bytes from global memory (wave-uniform base + per-lane 32-bit offset) straight into
// 1 KiB of consecutive LDS starting at the wave-uniform LDS address `lds_dst`.  Asynchronous (vmcnt).
__device__ __forceinline__ void load_1k_to_lds(uint32_t lane_offset, const char* base, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_dst), "v"(lane_offset), "s"(base)
               : "memory", "m0");
}
// The same with M0 (the LDS destination) left as the previous call set it: the instruction's immediate offset kOff is
// added to the LDS address and to the global address alike, so the caller passes a base that is kOff too low.
template <int kOff>
__device__ __forceinline__ void load_1k_to_lds_next(uint32_t lane_offset, const char* base_minus_off) {
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(lane_offset), "s"(base_minus_off), "n"(kOff) : "memory");
}

// Tiles [tile_begin, tile_begin + count) of the 256x256 tiling are covered.
//
// k_splits > 1 fills the chip during a last, partial round of tiles: a tile is shared by
// k_splits workgroups, each summing one contiguous range of K steps.  Every one of
// them stores its FP32 partial tile to `partials`, then takes a ticket from the tile's counter
// (zeroed by the decode pass of the same call); the workgroup that draws the last ticket adds the
// partials in split order - a fixed order, so the result does not depend on which workgroup
// finishes last - and stores the tile.  Nobody waits for anybody, so the scheme cannot deadlock
// whatever else shares the GPU.
template <bool kBf16Out>
__global__ __launch_bounds__(kThreads) void gemm_f16_kernel(const _Float16* __restrict__ A, const _Float16* __restrict__ B,
                                                            int64_t M, int64_t N, int64_t K, const float* __restrict__ a_ts,
                                                            const float* __restrict__ b_ts, void* __restrict__ Dv,
                                                            int64_t ldd, bool accumulate, int tiles_m, int tiles_n,
                                                            int tile_begin, int tile_count, int k_splits, float* partials,
                                                            unsigned int* tickets, bool a_ts_per_row, bool b_ts_per_row) {
  extern __shared__ __attribute__((aligned(16))) char lds[];

  // Workgroup -> tile: consecutive ids go to different XCDs (round robin over 8, one L2 each);
  // give every XCD a contiguous range of tiles, walked in bands of 8 tile rows.
  int wg = blockIdx.x, split = 0;
  if (k_splits > 1) {
    split = wg % k_splits;
    wg /= k_splits;
  }
  if ((tile_count & 7) == 0) wg = (wg & 7) * (tile_count >> 3) + (wg >> 3);
  const int tile_local = wg;
  const int pid = tile_begin + wg;
  constexpr int kBand = 8;
  const int band = pid / (kBand * tiles_n);
  const int band_rows = min(kBand, tiles_m - band * kBand);
  const int in_band = pid - band * kBand * tiles_n;
  const int tm = band * kBand + in_band % band_rows, tn = in_band / band_rows;
  const int64_t m0 = static_cast<int64_t>(tm) * TM, n0 = static_cast<int64_t>(tn) * TN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1, l16 = lane & 15, lq = lane >> 4;
  const int arow = wm * 128 + l16, brow = wn * 128 + l16;

  // Direct-load sources: instruction q of wavefront w fills rows w * 64 + 8 q .. + 7 of a tile (lane -> row lane / 8,
  // position lane % 8, i.e. chunk (lane % 8) ^ ((row >> 1) & 7); adding 8 q to the row leaves that term alone for even
  // q and flips its bit 2 for odd q).  Wave-uniform 64-bit base per 8-row block + one per-lane 32-bit offset for
  // even and one for odd q, shared by both operands (8 rows of K * 2 bytes: K < 2^21, checked on the host).  A block
  // past the end of an operand is replaced by the operand's last block (rows come in multiples of 16); it only
  // feeds outputs that are never stored.
  const int r0 = wave * 64 + (lane >> 3);
  const uint32_t c0 = static_cast<uint32_t>((lane & 7) ^ ((r0 >> 1) & 7)) * 16u;
  const uint32_t off_even = static_cast<uint32_t>(lane >> 3) * static_cast<uint32_t>(K * 2) + c0;
  const uint32_t off_odd = static_cast<uint32_t>(lane >> 3) * static_cast<uint32_t>(K * 2) + (c0 ^ 64u);
  const char* blk_a[8];
  const char* blk_b[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int64_t r = wave * 64 + q * 8;
    blk_a[q] = reinterpret_cast<const char*>(A) + (m0 + min<int64_t>(r, M - 8 - m0)) * K * 2;
    blk_b[q] = reinterpret_cast<const char*>(B) + (n0 + min<int64_t>(r, N - 8 - n0)) * K * 2;
  }
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));
  const uint32_t fill0 = lds0 + wave * 8192;   // this wavefront's 8 KiB of each operand tile
  // one of the 16 loads of K step kt into stage `stage`: q 0..7 A, 8..15 B
  auto issue_one = [&](int q, int kt, int stage) {
    const uint32_t dst = fill0 + stage * kStageBytes + (q < 8 ? 0 : kOperandBytes) + (q & 7) * 1024;
    load_1k_to_lds((q & 1) ? off_odd : off_even, (q < 8 ? blk_a[q & 7] : blk_b[q & 7]) + static_cast<int64_t>(kt) * kRowBytes, dst);
  };
  // The loads inside the loop, one instruction each where the prologue's form takes three plus address arithmetic
  // (a single wavefront per SIMD issues in order: what it spends on anything else, the matrix pipe waits):
  //   - the K step enters through the per-lane offsets, advanced once per step (ve, vo below), so the sixteen 64-bit
  //     row-block bases stay constant in scalar registers;
  //   - M0 (the LDS destination) is written once per four loads; loads q % 4 = 1, 2, 3 reach the next KiB through
  //     the instruction's immediate offset, which moves the LDS and the global address alike, hence bases that are
  //     (q % 4) KiB too low.
  const char* adj_a[8];
  const char* adj_b[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    adj_a[q] = blk_a[q] - (q & 3) * 1024;
    adj_b[q] = blk_b[q] - (q & 3) * 1024;
  }
  uint32_t ve = 0, vo = 0;   // off_even / off_odd + the byte offset of the K step being fetched
  auto issue_in_loop = [&](auto qc, int stage) {
    constexpr int q = decltype(qc)::value;
    const uint32_t voff = (q & 1) ? vo : ve;
    const char* base = q < 8 ? adj_a[q & 7] : adj_b[q & 7];
    if constexpr ((q & 3) == 0)
      load_1k_to_lds(voff, base, fill0 + stage * kStageBytes + (q < 8 ? 0 : kOperandBytes) + (q & 4) * 1024);
    else
      load_1k_to_lds_next<(q & 3) * 1024>(voff, base);
  };
  // fragment addresses in stage 0: first / second 32 k of the step
  const uint32_t a_lo = lds0 + swz(arow, lq), a_hi = lds0 + swz(arow, 4 + lq);
  const uint32_t b_lo = lds0 + kOperandBytes + swz(brow, lq), b_hi = lds0 + kOperandBytes + swz(brow, 4 + lq);

  float4v acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

  const int KT = static_cast<int>(K / TK);
  const int kt_begin = static_cast<int>(static_cast<int64_t>(KT) * split / k_splits);
  const int kt_end = static_cast<int>(static_cast<int64_t>(KT) * (split + 1) / k_splits);   // > kt_begin: KT >= k_splits
  static_for<0, 16>([&](auto q) { issue_one(decltype(q)::value, kt_begin, 0); });
  static_for<0, 16>([&](auto q) { issue_one(decltype(q)::value, min(kt_begin + 1, kt_end - 1), 1); });
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  Frags f0, f1;
  static_for<0, 16>([&](auto q) { read_frag<decltype(q)::value>(f0, a_lo, b_lo); });
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const uint32_t cur = ((kt - kt_begin) & 1) * kStageBytes, nxt = cur ^ kStageBytes;
    // Past the end the last K step is fetched again, into a buffer nobody reads any more: no branches in the loop.
    const int kt2 = min(kt + 2, kt_end - 1);
    ve = off_even + static_cast<uint32_t>(kt2) * kRowBytes;
    vo = off_odd + static_cast<uint32_t>(kt2) * kRowBytes;
    static_for<0, 64>([&](auto ic) {
      constexpr int n = decltype(ic)::value;
      mfma(acc[n >> 3][n & 7], f0.b[n & 7], f0.a[n >> 3]);
      if constexpr ((n & 3) == 1) read_frag<(n >> 2)>(f1, a_hi + cur, b_hi + cur);
    });
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    static_for<0, 64>([&](auto ic) {
      constexpr int n = decltype(ic)::value;
      mfma(acc[n >> 3][n & 7], f1.b[n & 7], f1.a[n >> 3]);
      if constexpr ((n & 3) == 1) read_frag<(n >> 2)>(f0, a_lo + nxt, b_lo + nxt);
      if constexpr ((n & 3) == 3) issue_in_loop(std::integral_constant<int, (n >> 2)>{}, (kt - kt_begin) & 1);
    });
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  // The trailing global->LDS loads must have landed before LDS is reused or the wavefront ends; the MFMA results
  // must have left the pipe before ordinary instructions read the accumulators (the compiler cannot see into the
  // assembly statements to insert these wait states itself).
  asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");
  __syncthreads();

  if (k_splits > 1) {
    // Partial tile in fragment order: float4 number (i * 8 + j) * 256 + tid.
    float4v* mine = reinterpret_cast<float4v*>(partials) +
                    (static_cast<int64_t>(tile_local) * k_splits + split) * (TM * TN / 4) + tid;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) mine[(i * 8 + j) * kThreads] = acc[i][j];
    // Publish: the barrier waits for every wavefront's stores to reach L2; then one thread makes
    // them visible device-wide (one L2 write-back per workgroup instead of one per wavefront),
    // draws the ticket and, if it is the last one, discards stale cached lines before anyone reads.
    __syncthreads();
    unsigned int* flag = reinterpret_cast<unsigned int*>(lds);   // LDS is free: the loop ended with a barrier
    if (tid == 0) {
      __threadfence();
      const unsigned int ticket = atomicAdd(tickets + tile_local, 1u);
      if (ticket == static_cast<unsigned int>(k_splits - 1)) __threadfence();
      *flag = ticket;
    }
    __syncthreads();
    if (*flag != static_cast<unsigned int>(k_splits - 1)) return;
    const float4v* all = reinterpret_cast<const float4v*>(partials) +
                         static_cast<int64_t>(tile_local) * k_splits * (TM * TN / 4) + tid;
    // acc = ((p0 + p1) + p2) + ...: every partial is fetched with 16 independent loads in flight.
    for (int sp = 0; sp < k_splits; ++sp) {
      const float4v* part = all + static_cast<int64_t>(sp) * (TM * TN / 4);
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        float4v t[2][8];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 8; ++j) t[i][j] = part[((h * 2 + i) * 8 + j) * kThreads];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[h * 2 + i][j] = sp == 0 ? t[i][j] : acc[h * 2 + i][j] + t[i][j];
      }
    }
  }

  // Tensor-level decode scales on the finished sums (App. B.3, after Eq. 5).
  const TensorScales out_scale{a_ts, b_ts, a_ts_per_row, b_ts_per_row};
  const int Mt = static_cast<int>(M - m0 < TM ? M - m0 : TM);
  const int Nt = static_cast<int>(N - n0 < TN ? N - n0 : TN);
  store_wave_block<kBf16Out>(acc, out_scale, Dv, ldd, accumulate, m0 + wm * 128, n0 + wn * 128, Mt - wm * 128, Nt - wn * 128,
                             lane);
}

}  // namespace

// Workspace: [A as FP16][B as FP16][256 tickets][split-K partial tiles], each part 256-byte aligned.
constexpr int kCUs = 256;
constexpr size_t kTicketBytes = kCUs * sizeof(unsigned int);
constexpr size_t kPartialTileBytes = static_cast<size_t>(TM) * TN * sizeof(float);

// How the last, partial round of 256x256 tiles is run: `tail` tiles (0 = there is none to treat
// specially) shared by `splits` workgroups each.
struct TailPlan {
  int tail, splits;
};

static TailPlan plan_tail(int64_t M, int64_t N, int64_t K) {
  const int64_t tiles = ((M + TM - 1) / TM) * ((N + TN - 1) / TN);
  TailPlan p{static_cast<int>(tiles % kCUs), 1};
  if (tiles < kCUs || p.tail == 0) return TailPlan{0, 1};
  const int64_t KT = K / TK;
  while (p.splits < 8 && p.tail * (p.splits * 2) <= kCUs && KT / (p.splits * 2) >= 8) p.splits *= 2;
  if (p.splits == 1) p.tail = 0;
  return p;
}

// FP16 bytes of the operands that still have to be decoded into the workspace (rows_a / rows_b: 0 for an operand the
// caller has decoded beforehand)
static size_t operand_bytes(int64_t rows_a, int64_t rows_b, int64_t K) {
  const size_t b = static_cast<size_t>(rows_a + rows_b) * static_cast<size_t>(K) * 2;
  return (b + 255) & ~static_cast<size_t>(255);
}

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  const TailPlan p = plan_tail(M, N, K);
  return operand_bytes(M, N, K) + kTicketBytes + static_cast<size_t>(p.tail) * p.splits * kPartialTileBytes;
}

static size_t workspace_need(const GemmArgs& g) {
  const TailPlan p = plan_tail(g.a.outer, g.b.outer, g.K);
  return operand_bytes(g.a.fp16 ? 0 : g.a.outer, g.b.fp16 ? 0 : g.b.outer, g.K) + kTicketBytes +
         static_cast<size_t>(p.tail) * p.splits * kPartialTileBytes;
}

bool gemm_two_pass_usable(const GemmArgs& g) {
  return g.workspace && g.workspace_bytes >= workspace_need(g) && (g.K % TK) == 0 &&
         reinterpret_cast<uintptr_t>(g.a.fp16) % 16 == 0 && reinterpret_cast<uintptr_t>(g.b.fp16) % 16 == 0 &&
         g.K < (int64_t{1} << 21) &&   // the kernel's 32-bit byte offsets inside a 256-row tile
         reinterpret_cast<uintptr_t>(g.workspace) % 256 == 0 && reinterpret_cast<uintptr_t>(g.a.codes) % 16 == 0 &&
         reinterpret_cast<uintptr_t>(g.b.codes) % 16 == 0 && reinterpret_cast<uintptr_t>(g.a.scales) % 2 == 0 &&
         reinterpret_cast<uintptr_t>(g.b.scales) % 2 == 0;
}

#define NVFP4_LAUNCH_F16(BF16)                                                                                    \
  do {                                                                                                            \
    static PerDeviceOnce once;                                                                                    \
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&gemm_f16_kernel<BF16>), kLdsBytes, once); \
    if (e != hipSuccess) return e;                                                                                \
    hipLaunchKernelGGL((gemm_f16_kernel<BF16>), dim3(wgs), dim3(kThreads), kLdsBytes, s, a16, b16,                   \
                       g.a.outer, g.b.outer, g.K, g.a.ts, g.b.ts, g.d, g.ldd, g.accumulate, tiles_m, tiles_n,     \
                       tile_begin, tile_count, k_splits, partials, tickets, g.a.ts_per_row != 0, g.b.ts_per_row != 0);    \
  } while (0)

static hipError_t launch_f16(bool bf16_out, const _Float16* a16, const _Float16* b16, const GemmArgs& g, int tiles_m,
                             int tiles_n, int tile_begin, int tile_count, int k_splits, float* partials,
                             unsigned int* tickets, hipStream_t s) {
  const unsigned wgs = static_cast<unsigned>(tile_count) * static_cast<unsigned>(k_splits);
  if (bf16_out) NVFP4_LAUNCH_F16(true); else NVFP4_LAUNCH_F16(false);
  return hipGetLastError();
}
#undef NVFP4_LAUNCH_F16

hipError_t launch_predecode(const Operand& op, int64_t K, void* fp16_out, hipStream_t s) {
  const int64_t n8 = op.outer * K / 8;
  hipLaunchKernelGGL(decode_f16_kernel, dim3(static_cast<unsigned>((n8 + 256 * kDecodeUnroll - 1) / (256 * kDecodeUnroll))), dim3(256), 0, s,
                     op.codes, op.scales, n8, static_cast<_Float16*>(fp16_out), op.codes, op.scales, int64_t{0},
                     static_cast<_Float16*>(fp16_out), static_cast<unsigned int*>(nullptr));
  return hipGetLastError();
}

hipError_t launch_gemm_two_pass(const GemmArgs& g, hipStream_t s) {
  const int64_t M = g.a.outer, N = g.b.outer, K = g.K;
  // Workspace: [A as FP16 unless decoded beforehand][B likewise][tickets][partial tiles]
  char* ws = static_cast<char*>(g.workspace);
  const int64_t rows_a = g.a.fp16 ? 0 : M, rows_b = g.b.fp16 ? 0 : N;
  _Float16* a_ws = reinterpret_cast<_Float16*>(ws);
  _Float16* b_ws = a_ws + rows_a * K;
  const _Float16* a16 = g.a.fp16 ? static_cast<const _Float16*>(g.a.fp16) : a_ws;
  const _Float16* b16 = g.b.fp16 ? static_cast<const _Float16*>(g.b.fp16) : b_ws;
  unsigned int* tickets = reinterpret_cast<unsigned int*>(ws + operand_bytes(rows_a, rows_b, K));
  float* partials = reinterpret_cast<float*>(ws + operand_bytes(rows_a, rows_b, K) + kTicketBytes);
  // One launch decodes what is still to decode and zeroes the tickets (with both operands decoded beforehand it is one
  // workgroup that only does the latter).
  const int64_t na = rows_a * K / 8, nb = rows_b * K / 8;   // a_n8 is a multiple of 256 only if M*K is a multiple of 2048; the kernel does not need it
  const int64_t nwg = (na + nb + 256 * kDecodeUnroll - 1) / (256 * kDecodeUnroll);
  hipLaunchKernelGGL(decode_f16_kernel, dim3(static_cast<unsigned>(nwg > 0 ? nwg : 1)), dim3(256), 0, s, g.a.codes,
                     g.a.scales, na, a_ws, g.b.codes, g.b.scales, nb, b_ws, tickets);
  const int tiles_m = static_cast<int>((M + TM - 1) / TM), tiles_n = static_cast<int>((N + TN - 1) / TN);
  const int tiles = tiles_m * tiles_n;
  // One 256x256 tile keeps one CU busy (its LDS fits one workgroup).  Whole rounds of kCUs tiles
  // run as they are; a last partial round that fills at most half the chip is split along K.
  const TailPlan p = plan_tail(M, N, K);
  const int full = tiles - p.tail;
  hipError_t e = hipSuccess;
  if (full > 0) e = launch_f16(g.out_bf16, a16, b16, g, tiles_m, tiles_n, 0, full, 1, nullptr, nullptr, s);
  if (e == hipSuccess && p.tail > 0)
    e = launch_f16(g.out_bf16, a16, b16, g, tiles_m, tiles_n, full, p.tail, p.splits, partials, tickets, s);
  return e;
}

}  // namespace nvfp4
