// Two-pass form of the block-scaled GEMM (App. B.3 Eq. 5) for gfx950, used when
// the caller lends a workspace:
//   pass 1  decode both NVFP4 operands to FP16, value * block_scale (exact: the
//           product has at most 6 significant bits), into the workspace, in the
//           order pass 2 loads them;
//   pass 2  a plain FP16 x FP16 -> FP32 MFMA GEMM whose main loop has no VALU
//           work but address increments: tiles go from global memory straight
//           into LDS (global_load_lds_dwordx4), fragments come from LDS,
//           16x16x32 MFMAs (measured under the chip's power limit: a
//           register-only loop of v_mfma_f32_16x16x32_f16 sustains 12-20 % more
//           flop/s than one of v_mfma_f32_32x32x16_f16 on the same operand
//           values); a workgroup runs its tiles as one stream of K steps;
//   pass 3  only for a last, partial round of tiles, which pass 2 splits along
//           K: the sum of the partial tiles.
// Why: decoding inside the GEMM loop costs about one VALU instruction per
// element, and VALU instructions co-issued with MFMAs take matrix-pipe time
// (measured: the fused kernel runs at 1.0-1.07 PFLOP/s, this route at 1.5-1.6
// in the GEMM proper, the decode pass adding 5-8 % of its time).
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

// Layout of a decoded operand ([outer, K] elements, outer a multiple of 16, K of 64): the piece the GEMM loads with
// one instruction and reads back as one MFMA fragment -- 16 rows x 32 k = 1 KiB -- is contiguous, the K steps of a
// 16-row block follow each other, and inside a piece the 16-byte chunks (8 k of one row) are in fragment order, the
// lane's order (lane l of an MFMA operand holds chunk l / 16 of row l % 16):
//   byte address of element (r, k) = ((r / 16) * (K / 32) + k / 32) * 1024 + (((k % 32) / 8) * 16 + r % 16) * 16 + (k % 8) * 2.
// So a load instruction reads 1 KiB of consecutive addresses into 1 KiB of consecutive LDS, and a fragment read is
// 1 KiB of consecutive LDS, lane l its bytes 16 l .. 16 l + 15: no bank conflicts, no swizzle.  (Measured with 8-row x
// 64-k pieces against rows of K * 2 bytes -- 8 separate 128-byte pieces per instruction, a stride that puts the
// pieces of all 256 tile rows into few cache channels: the GEMM's K step took 5-10 % less time on the three 12B
// shapes, same process, same data, identical results.)
//
// The decode pass: a workgroup takes a 16-row block x 512 k.  It reads the block's codes and scales row by row (256
// and 32 contiguous bytes per row), passes them through LDS, and writes 16 pieces of FP16 in output order, a thread
// 16 bytes at a time, consecutive threads consecutive addresses -- so that both sides of the pass move whole cache
// lines.  Both operands are decoded by one launch: the 16-row blocks of B follow those of A in the grid.
constexpr int kDecodeK = 512;                           // k per workgroup
constexpr int kDecodeCodeRow = kDecodeK / 2 + 16;       // bytes per row of codes in LDS; the 16 keep 16 rows off each other's banks
constexpr int kDecodeScaleRow = kDecodeK / 16 + 4;      // likewise for the scales
__global__ __launch_bounds__(256) void decode_f16_kernel(const uint8_t* __restrict__ a_codes,
                                                         const uint8_t* __restrict__ a_scales, int a_blocks,
                                                         _Float16* __restrict__ a_out,
                                                         const uint8_t* __restrict__ b_codes,
                                                         const uint8_t* __restrict__ b_scales, int b_blocks,
                                                         _Float16* __restrict__ b_out, int64_t K) {
  __shared__ __attribute__((aligned(16))) uint8_t lds_codes[16 * kDecodeCodeRow];
  __shared__ __attribute__((aligned(4))) uint8_t lds_scales[16 * kDecodeScaleRow];
  // consecutive workgroups walk along K: they read consecutive pieces of the same 16 rows and write consecutive 16 KiB
  const int k_groups = static_cast<int>((K + kDecodeK - 1) / kDecodeK);
  int blk = static_cast<int>(blockIdx.x) / k_groups;
  const int k_group = static_cast<int>(blockIdx.x) - blk * k_groups;
  const bool in_a = blk < a_blocks;
  if (!in_a) blk -= a_blocks;
  if (!in_a && blk >= b_blocks) return;
  const uint8_t* codes = in_a ? a_codes : b_codes;
  const uint8_t* scales = in_a ? a_scales : b_scales;
  uint4* out = reinterpret_cast<uint4*>(in_a ? a_out : b_out);
  const int t = static_cast<int>(threadIdx.x);
  const int64_t k0 = static_cast<int64_t>(k_group) * kDecodeK;
  {
    // codes: thread -> row t / 16, 32 elements (16 bytes) at k = k0 + 32 (t % 16)
    const int row = t >> 4, piece = t & 15;
    const int64_t k = k0 + piece * 32;
    if (k < K)
      *reinterpret_cast<uint4*>(lds_codes + row * kDecodeCodeRow + piece * 16) =
          *reinterpret_cast<const uint4*>(codes + ((static_cast<int64_t>(blk) * 16 + row) * K + k) / 2);
    // scales: threads 0..127 -> row t / 8, the four scale bytes of the 64 k from k0 + 64 (t % 8)
    if (t < 128) {
      const int srow = t >> 3, j = t & 7;
      if (k0 + j * 64 < K)
        *reinterpret_cast<uint32_t*>(lds_scales + srow * kDecodeScaleRow + j * 4) =
            *reinterpret_cast<const uint32_t*>(scales + ((static_cast<int64_t>(blk) * 16 + srow) * K + k0 + j * 64) / 16);
    }
  }
  __syncthreads();
  const int64_t pieces_per_block = K / 32;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    // 16-byte chunk number o of the workgroup's output: piece o / 64 (32 k each), chunk (o / 16) % 4 of it, row o % 16
    const int o = u * 256 + t;
    const int piece = o >> 6, chunk = (o >> 4) & 3, r16 = o & 15;
    if (k0 + piece * 32 >= K) break;
    const uint32_t c = *reinterpret_cast<const uint32_t*>(lds_codes + r16 * kDecodeCodeRow + piece * 16 + chunk * 4);
    const uint32_t s4 = *reinterpret_cast<const uint32_t*>(lds_scales + r16 * kDecodeScaleRow + (piece >> 1) * 4);
    const uint32_t scale = (s4 >> ((((piece & 1) * 2) + (chunk >> 1)) * 8)) & 0xffu;
    out[(static_cast<int64_t>(blk) * pieces_per_block + k0 / 32 + piece) * 64 + chunk * 16 + r16] = dec8(c, scale_h2(scale));
  }
}

// ---------------------------------------------------------------- pass 2: FP16 GEMM
// 256 x 256 outputs per workgroup, 256 threads = 4 wavefronts (2 x 2), one per SIMD,
// each 128 x 128 outputs as 8 x 8 MFMA 16x16 blocks: 256 accumulator registers, which live in
// the accumulation half of the register file, and 16 fragment loads per 64 MFMAs (a 128 x 64
// wave tile needs 12 per 32).  LDS is a ring of four stages of 32 k: (A tile, B tile) as 16 + 16 pieces of
// 16 rows x 32 k, 32 KiB a stage.  A stage is filled by direct global->LDS loads: one instruction moves 64 lanes x 16
// bytes, one piece of the decoded operand, into 1 KiB of consecutive LDS, which is one MFMA fragment in lane order.
//
// With one wavefront per SIMD nothing else can fill the matrix pipe while this one waits, so the
// loop is software-pipelined and its instruction order is fixed by hand (inline
// assembly keeps the compiler from regrouping it; measured 1.18 against 1.06 PFLOP/s for the
// 8-wavefront form on the same operands, at a lower clock: the chip's power limit sets the speed,
// and this form moves a third less data from LDS per flop).  Stage g:
//   64 MFMAs on the fragments read during stage g - 1; after every fourth, one of the 16 fragment loads of stage
//   g + 1; after every eighth, one of the wavefront's 8 global->LDS loads of stage g + 4 into the buffer of stage g,
//   which nobody reads any more
//   wait      own fragment loads back; own global->LDS loads of stage g + 2 landed (those of g + 3 and g + 4 may
//             still be on their way); barrier: every wavefront holds stage g + 1 in registers, stage g + 2 is complete
// so a load has three to four stages -- some 1.5 us -- to arrive in.
constexpr int TM = 256, TN = 256, TK = 64;       // TK: the unit K is split and counted in, two stages
constexpr int kThreads = 256;
constexpr int kStageK = 32;
constexpr int kPieceBytes = 16 * kStageK * 2;           // what one load instruction moves: 16 rows x 32 k, 1 KiB, contiguous in the decoded operand
constexpr int kOperandBytes = (TM / 16) * kPieceBytes;  // 16 KiB
constexpr int kStageBytes = 2 * kOperandBytes;          // 32 KiB
constexpr int kStages = 4;
constexpr int kLdsBytes = kStages * kStageBytes;

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

// Fragment q of a 16-fragment set: 0..7 = A rows i * 16, 8..15 = B rows j * 16: one piece each.
template <int q>
__device__ __forceinline__ void read_frag(Frags& f, uint32_t a_addr, uint32_t b_addr) {
  if constexpr (q < 8) lds_read16<q * kPieceBytes>(f.a[q], a_addr);
  else lds_read16<(q - 8) * kPieceBytes>(f.b[q - 8], b_addr);
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

// The first MFMA of an accumulator in a work item: C = 0, so the 256 accumulation registers are never cleared.
__device__ __forceinline__ void mfma_first(float4v& acc, const half8v& b, const half8v& a) {
  asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, 0" : "=a"(acc) : "v"(b), "v"(a));
}

// A wavefront's output stage issues 32 (bf16) or 64 (FP32) stores for a full 256 x 256 tile (store_wave_block: 16 bytes
// per lane and instruction).  Three quarters of them: the number of its memory operations that may still be
// outstanding when the loads issued before it are needed, with a margin against a store more or less.
template <bool kBf16Out>
constexpr int kTileStores = kBf16Out ? 24 : 48;

// Tiles [tile_begin, tile_begin + tile_count) of the 256x256 tiling are covered.
//
// k_splits == 1: a workgroup takes tiles blockIdx.x, blockIdx.x + gridDim.x, ... of the launch (the host launches one
// workgroup per CU when there are more tiles than CUs) and runs them as ONE stream of stages: the loads issued during a
// tile's last four stages already fetch the next tile's first four, so that the pipeline neither drains nor refills at
// a tile boundary -- what remains there is reading the 256 sums out, scaling, converting and issuing the stores,
// which then drain under the next tile's MFMAs (measured with timestamps in the one-tile-per-workgroup form: 4.2 us
// of pipeline fill, 5.5 us of output stage, most of it waiting for the stores of all CUs at once, and 0.6 us between
// workgroups, per 118 us of main loop at K = 5120).  Needs K >= 4 stages (2 K steps of 64); the host launches one workgroup per tile
// otherwise.
//
// k_splits > 1 (one work item per workgroup) fills the chip during a last, partial round of tiles: a tile is shared by
// k_splits workgroups, each summing one contiguous range of K steps and storing its FP32 partial tile to
// `partials`; splitk_sum_kernel, launched behind this one, adds the partials in split order and stores the tiles.
// (The sum used to be done here, by whichever workgroup of a tile finished last, found by a ticket counter: by
// timestamps inside the kernel, of the 127 us such a launch took on 64 tiles x 4 splits at K = 8192, the K steps
// were 48, the partial stores 7, the device-wide fence and the ticket 10, and one workgroup fetching and adding the
// 1 MiB that four XCDs had written 50 -- with 16 loads in flight per thread, and 90 with 64.)
// kRowScales: an operand carries a tensor-level scale per row (uniform over a launch, and a different output stage).
// kSplit: k_splits > 1; the output stage is the store of the partial tile (kBf16Out and kRowScales are false then).
template <bool kBf16Out, bool kRowScales, bool kSplit>
__global__ __launch_bounds__(kThreads) void gemm_f16_kernel(const _Float16* __restrict__ A, const _Float16* __restrict__ B,
                                                            int64_t M, int64_t N, int64_t K, const float* __restrict__ a_ts,
                                                            const float* __restrict__ b_ts, void* __restrict__ Dv,
                                                            int64_t ldd, bool accumulate, int tiles_m, int tiles_n,
                                                            int tile_begin, int tile_count, int k_splits, float* partials,
                                                            bool a_ts_per_row, bool b_ts_per_row) {
  extern __shared__ __attribute__((aligned(16))) char lds[];

  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) >> 6);

  // Work item -> tile: consecutive workgroup ids go to different XCDs (round robin over 8, one L2 each);
  // give every XCD a contiguous range of tiles, walked in bands of 8 tile rows.  (With one workgroup per CU the ids
  // of a later round continue the first round's, 8 | gridDim.x, so the low three bits stay the XCD.)
  auto locate = [&](int wg, int& tm, int& tn) -> int {
    if ((tile_count & 7) == 0) wg = (wg & 7) * (tile_count >> 3) + (wg >> 3);
    tile_coordinates(tile_begin + wg, tiles_m, tiles_n, tm, tn);
    return wg;   // the tile's number within the launch
  };

  // Direct-load sources: instruction q of wavefront w fills rows w * 64 + 16 q .. + 15 of a tile, which the decoded
  // operand holds as 1 KiB of consecutive bytes per stage, in LDS order (lane l: bytes 16 l .. 16 l + 15).  An address
  // is a wave-uniform 64-bit base per operand, which holds the tile and the stage being fetched, plus a per-lane
  // 32-bit offset per instruction (256 rows of K * 2 bytes: K < 2^21, checked on the host), which holds the 16-row
  // block and does not change within a tile: moving on by a stage is two scalar additions per operand.  (Every
  // vector instruction between two MFMAs costs: with the stage added to the 8 per-lane offsets instead, the three
  // 12B GEMM calls took 2 % longer.)  A block past the end of an operand is replaced by the operand's last block
  // (rows come in multiples of 16); it only feeds outputs that are never stored.
  // One instruction per load inside the loop (a single wavefront per SIMD issues in order: what it spends on anything
  // else, the matrix pipe waits): M0, the LDS destination, is written once per four loads; loads q % 4 = 1, 2, 3 reach
  // the next KiB through the instruction's immediate offset, which moves the LDS and the global address alike, so
  // the bases sit 3 KiB low and the offsets make up for what the immediate does not add.
  //
  // What depends on the lane is worked out once per tile, from a lane number asked for on the spot: values the
  // compiler could keep from before the first tile would have to live through every output stage, which needs the
  // registers itself, and end up in scratch memory, to be fetched back inside the K steps.
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));
  uint32_t lane_bytes = 0;          // the lane's part of a load offset
  uint32_t a_frag = 0, b_frag = 0;  // the lane's 16 bytes of the wavefront's first A / B fragment in ring buffer 0
  auto lane_setup = [&]() {
    lane_bytes = static_cast<uint32_t>(lane_id()) * 16u;
    a_frag = lds0 + (wave >> 1) * (8 * kPieceBytes) + lane_bytes;
    b_frag = lds0 + kOperandBytes + (wave & 1) * (8 * kPieceBytes) + lane_bytes;
  };
  lane_setup();
  const char* base_a = nullptr;
  const char* base_b = nullptr;
  uint32_t voff[8];   // q 0..3 A, 4..7 B
  // Point the loads at stage st (32 k) of tile (tm, tn).
  auto aim = [&](int tm, int tn, int st) {
    const int64_t m_first = static_cast<int64_t>(tm) * TM, n_first = static_cast<int64_t>(tn) * TN;
    base_a = reinterpret_cast<const char*>(A) + m_first * K * 2 + (st - 3) * kPieceBytes;
    base_b = reinterpret_cast<const char*>(B) + n_first * K * 2 + (st - 3) * kPieceBytes;
    // 16-row blocks counted from the tile's first; a block's stages are K / 32 KiB
    const uint32_t last_a = static_cast<uint32_t>(M - 16 - m_first) >> 4, last_b = static_cast<uint32_t>(N - 16 - n_first) >> 4;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t blk = static_cast<uint32_t>(wave * 4 + q);
      const uint32_t fixed = static_cast<uint32_t>(3 - q) * 1024u;
      voff[q] = lane_bytes + min(blk, last_a) * static_cast<uint32_t>(K * 32) + fixed;
      voff[4 + q] = lane_bytes + min(blk, last_b) * static_cast<uint32_t>(K * 32) + fixed;
    }
  };
  const uint32_t fill0 = lds0 + wave * (4 * kPieceBytes);   // this wavefront's 4 KiB of each operand tile
  // load q of the wavefront's 8 that fill ring buffer `buf`
  auto issue = [&](auto qc, uint32_t buf) {
    constexpr int q = decltype(qc)::value;
    const char* base = q < 4 ? base_a : base_b;
    if constexpr ((q & 3) == 0) load_1k_to_lds(voff[q], base, fill0 + buf * kStageBytes + (q < 4 ? 0 : kOperandBytes));
    else load_1k_to_lds_next<(q & 3) * 1024>(voff[q], base);
  };

  const int KT = static_cast<int>(K / TK);
  const int items = tile_count * k_splits;
  int item = blockIdx.x;   // < items: the host launches at most that many workgroups
  int tm = 0, tn = 0;
  const int split = item % k_splits;   // k_splits > 1: one work item per workgroup
  const int tile_local = locate(item / k_splits, tm, tn);
  int kt_begin = static_cast<int>(static_cast<int64_t>(KT) * split / k_splits);
  int kt_end = static_cast<int>(static_cast<int64_t>(KT) * (split + 1) / k_splits);   // > kt_begin: KT >= k_splits
  // The stage the loads were last pointed at: they run four stages ahead of the MFMAs.
  int fetch_st = 2 * kt_begin;
  aim(tm, tn, fetch_st);
  static_for<0, 8>([&](auto q) { issue(q, 0); });
#pragma unroll
  for (uint32_t buf = 1; buf < kStages; ++buf) {
    if (fetch_st + 1 < 2 * kt_end) {   // (an item of two stages fetches its last three times)
      ++fetch_st;
      base_a += kPieceBytes;
      base_b += kPieceBytes;
    }
    static_for<0, 8>([&](auto q) { issue(q, buf); });
  }
  asm volatile("s_waitcnt vmcnt(16)" ::: "memory");   // the first two stages
  __builtin_amdgcn_s_barrier();

  Frags f0, f1;
  float4v acc[8][8];
  uint32_t g = 0;               // stages done so far; stage g lives in ring buffer g % 4
  bool stores_behind = false;   // the previous tile's kTileStores stores were issued after the loads now in flight
  for (;;) {
    // The tile's first fragments.  (After a tile of the same stream its last stage has read them already; they are read
    // again so that the output stage had their registers to work with.)  The barrier: the first stage loads into the
    // buffer these came from.
    {
      const uint32_t cur = (g & 3u) * kStageBytes;
      static_for<0, 16>([&](auto q) { read_frag<decltype(q)::value>(f0, a_frag + cur, b_frag + cur); });
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    // The next tile of this workgroup, if any: its stages follow this tile's without a break (k_splits == 1 then).
    const int next_item = item + static_cast<int>(gridDim.x);
    const bool has_next = next_item < items;
    int next_tm = 0, next_tn = 0;
    if (has_next) locate(next_item, next_tm, next_tn);
    const int st_end = 2 * kt_end;

    // One stage on the fragments in `fc`, reading the next stage's into `fn`.  kFirst: the item's first (accumulators
    // start from zero); kRelaxed: one of its first two (the stores of the tile before may still be in flight behind
    // the loads this stage waits for).
    auto stage = [&](auto first_tag, auto relaxed_tag, Frags& fc, Frags& fn) {
      constexpr bool kFirst = decltype(first_tag)::value, kRelaxed = decltype(relaxed_tag)::value;
      const uint32_t buf = g & 3u, nxt = ((g + 1u) & 3u) * kStageBytes;
      // The loads move on one stage: within the tile, or to the next tile's stage 0, or, with nothing to follow, not at
      // all (the last stage is fetched again, into a buffer nobody reads any more: no branches around the loads).
      uint32_t advance = kPieceBytes;
      if (fetch_st + 1 < st_end) {
        ++fetch_st;
      } else {
        advance = 0;
        if (has_next) {
          fetch_st = 0;
          aim(next_tm, next_tn, 0);
        }
      }
      static_for<0, 64>([&](auto ic) {
        constexpr int n = decltype(ic)::value;
        if constexpr (kFirst) mfma_first(acc[n >> 3][n & 7], fc.b[n & 7], fc.a[n >> 3]);
        else mfma(acc[n >> 3][n & 7], fc.b[n & 7], fc.a[n >> 3]);
        if constexpr ((n & 3) == 1) read_frag<(n >> 2)>(fn, a_frag + nxt, b_frag + nxt);
        if constexpr (n == 3) base_a += advance;
        if constexpr (n == 35) base_b += advance;
        if constexpr ((n & 7) == 3) issue(std::integral_constant<int, (n >> 3)>{}, buf);
      });
      // Memory operations complete in issue order.  Behind the loads of stage g + 2 this wavefront has issued those of
      // g + 3 and g + 4, 8 each, and, across a tile boundary, the stores of the tile before.
      if (kRelaxed && stores_behind)
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(16 + kTileStores<kBf16Out> > 63 ? 63 : 16 + kTileStores<kBf16Out>) : "memory");
      else asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      ++g;
    };
    stage(std::true_type{}, std::true_type{}, f0, f1);
    stage(std::false_type{}, std::true_type{}, f1, f0);
    for (int kt = kt_begin + 1; kt < kt_end; ++kt) {
      stage(std::false_type{}, std::false_type{}, f0, f1);
      stage(std::false_type{}, std::false_type{}, f1, f0);
    }

    // Everything below is computed here, per tile: were the compiler to move the output stage's loop-invariant
    // address arithmetic in front of the stream, it would have to keep it in registers through the K steps, which
    // have none to spare.
    int wm = wave >> 1, wn = wave & 1;
    asm volatile("" : "+s"(wm), "+s"(wn));
    const int lane = lane_id(), tid = (wm * 2 + wn) * 64 + lane;
    // Tensor-level decode scales on the finished sums (App. B.3, after Eq. 5).
    const TensorScales out_scale{a_ts, b_ts, a_ts_per_row, b_ts_per_row};
    const int64_t m0 = static_cast<int64_t>(tm) * TM, n0 = static_cast<int64_t>(tn) * TN;
    const int Mt = static_cast<int>(M - m0 < TM ? M - m0 : TM);
    const int Nt = static_cast<int>(N - n0 < TN ? N - n0 : TN);
    // The MFMA results must have left the pipe before ordinary instructions read the accumulators (the compiler
    // cannot see into the assembly statements to insert these wait states itself).  With nothing to follow, the
    // trailing global->LDS loads must have landed before the wavefront ends; otherwise the next
    // tile's first two stages are in LDS by now and two more on their way there.
    if (has_next) {
      asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");
      __syncthreads();
    }

    if constexpr (kSplit) {   // has_next is false
      // Partial tile in fragment order: float4 number (i * 8 + j) * 256 + tid.
      float4v* mine = reinterpret_cast<float4v*>(partials) +
                      (static_cast<int64_t>(tile_local) * k_splits + split) * (TM * TN / 4) + tid;
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) mine[(i * 8 + j) * kThreads] = acc[i][j];
      return;
    } else {
      store_wave_block_impl<kBf16Out, kRowScales>(acc, out_scale, Dv, ldd, accumulate, m0 + wm * 128, n0 + wn * 128,
                                                  Mt - wm * 128, Nt - wn * 128, lane);
    }
    if (!has_next) break;
    stores_behind = Mt == TM && Nt == TN;   // every lane stored every block: the count is known
    item = next_item;
    tm = next_tm;
    tn = next_tn;
    kt_begin = 0;
    kt_end = KT;
    lane_setup();
    aim(tm, tn, fetch_st);
  }
}

// The sums over K of the tiles a split-K launch covered: one wavefront per tile, 128 x 128 block of it (the block one
// wavefront of gemm_f16_kernel holds, in the same register layout, which is the order the partial tiles are stored
// in) and 16 rows of that, sum = ((p0 + p1) + p2) + ... in split order, then the same output stage.  Many small
// workgroups: the partial tiles were written by other XCDs and every load of them is a long trip, so what counts is
// how many are in flight over the chip (with a wavefront per 128 x 128 block the sum of 64 tiles x 4 splits took 57 us).
template <bool kBf16Out, bool kRowScales>
__global__ __launch_bounds__(64) void splitk_sum_kernel(const float* __restrict__ partials, int k_splits, int64_t M, int64_t N,
                                                        const float* __restrict__ a_ts, const float* __restrict__ b_ts,
                                                        void* __restrict__ Dv, int64_t ldd, bool accumulate, int tiles_m,
                                                        int tiles_n, int tile_begin, bool a_ts_per_row, bool b_ts_per_row) {
  const int tile_local = static_cast<int>(blockIdx.x) >> 5, wave = (static_cast<int>(blockIdx.x) >> 3) & 3;
  const int i = static_cast<int>(blockIdx.x) & 7;
  const int lane = static_cast<int>(threadIdx.x), wm = wave >> 1, wn = wave & 1;
  int tm, tn;
  tile_coordinates(tile_begin + tile_local, tiles_m, tiles_n, tm, tn);
  // float4 number (i * 8 + j) * 256 + 64 wave + lane of a partial tile
  const float4v* all = reinterpret_cast<const float4v*>(partials) +
                       static_cast<int64_t>(tile_local) * k_splits * (TM * TN / 4) + i * 8 * kThreads + wave * 64 + lane;
  float4v sums[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) sums[j] = all[j * kThreads];
  for (int sp = 1; sp < k_splits; ++sp) {
    const float4v* part = all + static_cast<int64_t>(sp) * (TM * TN / 4);
    float4v t[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] = part[j * kThreads];
#pragma unroll
    for (int j = 0; j < 8; ++j) sums[j] = sums[j] + t[j];
  }
  const TensorScales ts{a_ts, b_ts, a_ts_per_row, b_ts_per_row};
  const int64_t m0 = static_cast<int64_t>(tm) * TM, n0 = static_cast<int64_t>(tn) * TN;
  const int Mt = static_cast<int>(M - m0 < TM ? M - m0 : TM);
  const int Nt = static_cast<int>(N - n0 < TN ? N - n0 : TN);
  const WaveBlockStore<kBf16Out, kRowScales> out(ts, Dv, ldd, accumulate, m0 + wm * 128, n0 + wn * 128, Mt - wm * 128,
                                                 Nt - wn * 128, lane);
  out.store_rows(sums, i, kRowScales ? out.row_scale(ts, m0 + wm * 128, i) : 0.0f);
}

}  // namespace

// Workspace: [A as FP16][B as FP16][split-K partial tiles], each part 256-byte aligned.
constexpr int kCUs = 256;
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
  return operand_bytes(M, N, K) + static_cast<size_t>(p.tail) * p.splits * kPartialTileBytes;
}

static size_t workspace_need(const GemmArgs& g) {
  const TailPlan p = plan_tail(g.a.outer, g.b.outer, g.K);
  return operand_bytes(g.a.fp16 ? 0 : g.a.outer, g.b.fp16 ? 0 : g.b.outer, g.K) +
         static_cast<size_t>(p.tail) * p.splits * kPartialTileBytes;
}

bool gemm_two_pass_usable(const GemmArgs& g) {
  // (With both operands decoded beforehand and no partial last round of tiles nothing is needed of the workspace.)
  const size_t need = workspace_need(g);
  const bool room = need == 0 || (g.workspace && g.workspace_bytes >= need && reinterpret_cast<uintptr_t>(g.workspace) % 256 == 0);
  return room && (g.K % TK) == 0 &&
         reinterpret_cast<uintptr_t>(g.a.fp16) % 16 == 0 && reinterpret_cast<uintptr_t>(g.b.fp16) % 16 == 0 &&
         g.K < (int64_t{1} << 21) &&   // the kernel's 32-bit byte offsets inside a 256-row tile
         reinterpret_cast<uintptr_t>(g.a.codes) % 16 == 0 &&
         reinterpret_cast<uintptr_t>(g.b.codes) % 16 == 0 && reinterpret_cast<uintptr_t>(g.a.scales) % 4 == 0 &&
         reinterpret_cast<uintptr_t>(g.b.scales) % 4 == 0;
}

#define NVFP4_LAUNCH_F16(BF16, ROWSCALES, SPLIT)                                                                  \
  do {                                                                                                            \
    static PerDeviceOnce once;                                                                                    \
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&gemm_f16_kernel<BF16, ROWSCALES, SPLIT>), kLdsBytes, once); \
    if (e != hipSuccess) return e;                                                                                \
    hipLaunchKernelGGL((gemm_f16_kernel<BF16, ROWSCALES, SPLIT>), dim3(wgs), dim3(kThreads), kLdsBytes, s, a16, b16, \
                       g.a.outer, g.b.outer, g.K, g.a.ts, g.b.ts, g.d, g.ldd, g.accumulate, tiles_m, tiles_n,     \
                       tile_begin, tile_count, k_splits, partials, g.a.ts_per_row != 0, g.b.ts_per_row != 0);      \
  } while (0)

// Tiles [tile_begin, tile_begin + tile_count); k_splits > 1: each shared by that many workgroups, summed by a second launch.
static hipError_t launch_f16(bool bf16_out, const _Float16* a16, const _Float16* b16, const GemmArgs& g, int tiles_m,
                             int tiles_n, int tile_begin, int tile_count, int k_splits, float* partials, hipStream_t s) {
  // More whole tiles than CUs: one workgroup per CU, each running its tiles as one stream of K steps.
  unsigned wgs = static_cast<unsigned>(tile_count) * static_cast<unsigned>(k_splits);
  if (k_splits == 1 && g.K / TK >= 2 && wgs > static_cast<unsigned>(kCUs)) wgs = kCUs;
  const bool row_scales = g.a.ts_per_row != 0 || g.b.ts_per_row != 0;
  if (k_splits > 1) {
    NVFP4_LAUNCH_F16(false, false, true);
    const dim3 grid(static_cast<unsigned>(tile_count) * 32);   // tile, 128 x 128 block, 16 rows
#define NVFP4_LAUNCH_SUM(BF16, ROWSCALES)                                                                              \
  hipLaunchKernelGGL((splitk_sum_kernel<BF16, ROWSCALES>), grid, dim3(64), 0, s, partials, k_splits, g.a.outer, g.b.outer, \
                     g.a.ts, g.b.ts, g.d, g.ldd, g.accumulate, tiles_m, tiles_n, tile_begin, g.a.ts_per_row != 0,      \
                     g.b.ts_per_row != 0)
    if (bf16_out) {
      if (row_scales) NVFP4_LAUNCH_SUM(true, true); else NVFP4_LAUNCH_SUM(true, false);
    } else {
      if (row_scales) NVFP4_LAUNCH_SUM(false, true); else NVFP4_LAUNCH_SUM(false, false);
    }
#undef NVFP4_LAUNCH_SUM
  } else if (row_scales) {
    if (bf16_out) NVFP4_LAUNCH_F16(true, true, false); else NVFP4_LAUNCH_F16(false, true, false);
  } else {
    if (bf16_out) NVFP4_LAUNCH_F16(true, false, false); else NVFP4_LAUNCH_F16(false, false, false);
  }
  return hipGetLastError();
}
#undef NVFP4_LAUNCH_F16

// Grid of the decode pass for `blocks` 16-row blocks: a workgroup per block and kDecodeK elements of K.  False
// if that is more than a grid can hold (operands beyond 2^44 elements).
static bool decode_grid(int64_t blocks, int64_t K, dim3* grid) {
  const int64_t n = blocks * ((K + kDecodeK - 1) / kDecodeK);
  if (n > 0x7fffffff) return false;
  *grid = dim3(static_cast<unsigned>(n));
  return true;
}

hipError_t launch_predecode(const Operand& op, int64_t K, void* fp16_out, hipStream_t s) {
  dim3 grid;
  if (!decode_grid(op.outer / 16, K, &grid)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(decode_f16_kernel, grid, dim3(256), 0, s, op.codes, op.scales,
                     static_cast<int>(op.outer / 16), static_cast<_Float16*>(fp16_out), op.codes, op.scales, 0,
                     static_cast<_Float16*>(fp16_out), K);
  return hipGetLastError();
}

hipError_t launch_gemm_two_pass(const GemmArgs& g, hipStream_t s) {
  const int64_t M = g.a.outer, N = g.b.outer, K = g.K;
  // Workspace: [A as FP16 unless decoded beforehand][B likewise][partial tiles]
  char* ws = static_cast<char*>(g.workspace);
  const int64_t rows_a = g.a.fp16 ? 0 : M, rows_b = g.b.fp16 ? 0 : N;
  _Float16* a_ws = reinterpret_cast<_Float16*>(ws);
  _Float16* b_ws = a_ws + rows_a * K;
  const _Float16* a16 = g.a.fp16 ? static_cast<const _Float16*>(g.a.fp16) : a_ws;
  const _Float16* b16 = g.b.fp16 ? static_cast<const _Float16*>(g.b.fp16) : b_ws;
  float* partials = reinterpret_cast<float*>(ws + operand_bytes(rows_a, rows_b, K));
  // One launch decodes what is still to decode.
  if (rows_a + rows_b > 0) {
    dim3 grid;
    if (!decode_grid((rows_a + rows_b) / 16, K, &grid)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(decode_f16_kernel, grid, dim3(256), 0, s, g.a.codes, g.a.scales, static_cast<int>(rows_a / 16), a_ws,
                       g.b.codes, g.b.scales, static_cast<int>(rows_b / 16), b_ws, K);
  }
  const int tiles_m = static_cast<int>((M + TM - 1) / TM), tiles_n = static_cast<int>((N + TN - 1) / TN);
  const int tiles = tiles_m * tiles_n;
  // One 256x256 tile keeps one CU busy (its LDS fits one workgroup).  Whole rounds of kCUs tiles
  // run as they are; a last partial round that fills at most half the chip is split along K.
  const TailPlan p = plan_tail(M, N, K);
  const int full = tiles - p.tail;
  hipError_t e = hipSuccess;
  if (full > 0) e = launch_f16(g.out_bf16, a16, b16, g, tiles_m, tiles_n, 0, full, 1, nullptr, s);
  if (e == hipSuccess && p.tail > 0)
    e = launch_f16(g.out_bf16, a16, b16, g, tiles_m, tiles_n, full, p.tail, p.splits, partials, s);
  return e;
}

}  // namespace nvfp4
