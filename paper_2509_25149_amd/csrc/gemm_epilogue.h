// What the 4-wavefront GEMM kernels for gfx950 share besides their loops: the walk over the 256 x 256 tiles, and the
// output stage: one wavefront's 128 x 128 block of FP32 sums,
// held as 8 x 8 results of 16x16 MFMAs (acc[i][j][r] = D[m = 16 i + (lane & 15)][n = 16 j + 4 (lane >> 4) + r]),
// times the tensor-level decode scales (App. B.3, after Eq. 5), to FP32 (optionally added into D) or bf16.
// Device code only.
#pragma once

#include "nvfp4_device.h"

namespace nvfp4 {

// row0 / col0: the block's first row / column in D; rows / cols: how many of its 128 x 128 exist (multiples of 16,
// possibly <= 0).  Stored from the registers, 64 contiguous bytes per row and instruction:
//   FP32  a lane writes its 4 consecutive columns of one row (16 bytes; the four lanes of a row 64 bytes);
//   bf16  a lane's 4 columns are only 8 bytes, so two neighbouring 16-column blocks are stored together: lanes
//         16 apart (column groups 4q.. and 4(q+1)..) trade halves with v_permlane16_swap_b32, after which an
//         even group holds 8 consecutive columns of the first block and an odd group 8 of the second.
// Ordinary stores throughout.  Non-temporal ones were measured both ways: for bf16 results (activations and their
// gradients, which the caller reads next) they made the amax pass behind Fprop a third faster (96 -> 62 us) but Fprop
// itself 4 % slower; for FP32 results (weight gradients) they took 3 us off the quantizer call that follows a Wgrad,
// but a wavefront's output stage issues them at two thirds of the rate (11.7 against 8.2 us for its 64 stores, by
// timestamps inside the kernel; the Wgrad call 1.359 against 1.347 ms).  A wavefront's stores leave at about 1 KiB per
// 150 cycles whatever else the chip does (the four wavefronts of a CU share one path to the L2: 128 KiB of bf16 per
// tile take 2.3 us, another 2.6 us go to reading, scaling and converting the 256 sums), so what bounds
// the output stage is what a wavefront has to issue, not memory bandwidth.  Must be called by all 64 lanes.  (Reordering the bf16 block through LDS into 256-byte row pieces was tried
// with ordinary stores and measured no faster.)
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));

// The lane's number within its wavefront, asked of the hardware at the place of the call: the compiler can neither
// move the question nor keep an earlier answer in a register.
__device__ __forceinline__ int lane_id() {
  int lane;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane));
  return lane;
}

// Tile number pid of the 256x256 tiling -> tile row and column: the tiles are walked in bands of 8 tile rows, column by
// column within a band.
__device__ __forceinline__ void tile_coordinates(int pid, int tiles_m, int tiles_n, int& tm, int& tn) {
  constexpr int kBand = 8;
  const int band = pid / (kBand * tiles_n);
  const int band_rows = min(kBand, tiles_m - band * kBand);
  const int in_band = pid - band * kBand * tiles_n;
  tm = band * kBand + in_band % band_rows;
  tn = in_band / band_rows;
}


// The two operands' tensor-level decode scales.  Per tensor: a[0] * b[0] for every output.  With a scale per row of an
// operand (App. B.1, last sentence) output (m, n) takes a[m] * b[n]: still constant along k, so still outside the sum.
struct TensorScales {
  const float* a;
  const float* b;
  bool a_per_row, b_per_row;
};

// scale of the four outputs (row m, columns n .. n + 3); m, n global indices inside the matrix (used by the kernels
// with small tiles; the 128 x 128 wave block below loads its scale vectors once)
__device__ __forceinline__ float4v scale4(const TensorScales& ts, float uniform, bool vec, bool in, int64_t m, int64_t n) {
  float4v s = {uniform, uniform, uniform, uniform};
  if (vec && in) {
    const float sa = ts.a[ts.a_per_row ? m : 0];
#pragma unroll
    for (int r = 0; r < 4; ++r) s[r] = sa * ts.b[ts.b_per_row ? n + r : 0];
  }
  return s;
}

// What a lane needs to know to store its part of a 128 x 128 block: kVec: an operand carries one scale per row; the
// lane's 8 x 4 columns (n = 16 j + 4 lq + r) then take their factors from sb, loaded once, and its 8 rows
// (m = 16 i + l16) one factor each.  Otherwise the product a[0] * b[0] serves every output.
// A lane's addresses are one pointer (its row l16, its first column) plus i * 16 rows plus a constant per j, which the
// stores carry as their immediate offsets.
template <bool kBf16Out, bool kVec>
struct WaveBlockStore {
  void* d;
  int64_t ldd, lane_first;
  int l16, nl, rows, cols;
  bool accumulate;
  float out_scale;
  float4v sb[kVec ? 8 : 1];

  __device__ __forceinline__ WaveBlockStore(const TensorScales ts, void* Dv, int64_t ldd_, bool accumulate_, int64_t row0, int64_t col0,
                                            int rows_, int cols_, int lane)
      : d(Dv), ldd(ldd_), l16(lane & 15), rows(rows_), cols(cols_), accumulate(accumulate_), out_scale(ts.a[0] * ts.b[0]) {
    const int lq = lane >> 4;
    // bf16: after the exchange a lane of an even column group holds 8 consecutive columns of block j, a lane of an odd
    // group 8 of block j + 1: column 16 j + nl, nl = 0, 16, 8, 24 for lq = 0 .. 3.
    nl = kBf16Out ? (lq & 1) * 16 + (lq >> 1) * 8 : lq * 4;
    lane_first = (row0 + l16) * ldd + col0 + nl;
    if (kVec) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (ts.b_per_row && j * 16 + lq * 4 < cols) {
          sb[kVec ? j : 0] = *reinterpret_cast<const float4v*>(ts.b + col0 + j * 16 + lq * 4);
        } else {
          const float b0 = ts.b[0];
          sb[kVec ? j : 0] = float4v{b0, b0, b0, b0};
        }
      }
    }
  }

  // the factor of the lane's row in 16-row block i (kVec only)
  __device__ __forceinline__ float row_scale(const TensorScales ts, int64_t row0, int i) const {
    return ts.a[ts.a_per_row && i * 16 + l16 < rows ? row0 + i * 16 + l16 : 0];
  }

  // The lane's 8 x 4 sums of 16-row block i: row m = 16 i + l16, columns 16 j + 4 lq + r.
  __device__ __forceinline__ void store_rows(const float4v (&sums)[8], int i, float sa) const {
    auto scale = [&](int j) -> float4v {
      if (kVec) return sb[kVec ? j : 0] * sa;
      return float4v{out_scale, out_scale, out_scale, out_scale};
    };
    const bool row_in = i * 16 + l16 < rows;
    if (kBf16Out) {
      uint16_t* d_row = static_cast<uint16_t*>(d) + lane_first + i * 16 * ldd;
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        const float4v va = sums[j] * scale(j), vb = sums[j + 1] * scale(j + 1);
        const uint32_t a0 = f32x2_to_bf16(va[0], va[1]), a1 = f32x2_to_bf16(va[2], va[3]);
        const uint32_t b0 = f32x2_to_bf16(vb[0], vb[1]), b1 = f32x2_to_bf16(vb[2], vb[3]);
        // first result: lanes of odd groups now hold the second block's dword of the group below; second result: lanes of
        // even groups now hold the first block's dword of the group above
        const auto s0 = __builtin_amdgcn_permlane16_swap(a0, b0, false, false);
        const auto s1 = __builtin_amdgcn_permlane16_swap(a1, b1, false, false);
        const u32x4v o = {s0[0], s1[0], s0[1], s1[1]};
        // columns come in multiples of 16, so the 8 columns are in or out together
        if (row_in && j * 16 + nl < cols) *reinterpret_cast<u32x4v*>(d_row + j * 16) = o;
      }
    } else {
      float* d_row = static_cast<float*>(d) + lane_first + i * 16 * ldd;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (row_in && j * 16 + nl < cols) {  // columns come in multiples of 16, so the 4 columns are in or out together
          float4v v = sums[j] * scale(j);
          float* p = d_row + j * 16;
          if (accumulate) v += *reinterpret_cast<const float4v*>(p);
          *reinterpret_cast<float4v*>(p) = v;
        }
      }
    }
  }
};

// A wavefront's whole 128 x 128 block.  (A variant without the predicates for blocks that exist whole measured no
// faster.)  A kernel should contain this once: where a second use of the sums sits in another branch, the compiler
// reads all 256 out of the accumulation registers ahead of the branch, into registers it does not have.
template <bool kBf16Out, bool kVec>
__device__ __forceinline__ void store_wave_block_impl(float4v (&acc)[8][8], const TensorScales ts, void* __restrict__ Dv, int64_t ldd,
                                                      bool accumulate, int64_t row0, int64_t col0, int rows, int cols, int lane) {
  const WaveBlockStore<kBf16Out, kVec> out(ts, Dv, ldd, accumulate, row0, col0, rows, cols, lane);
  float sa[kVec ? 8 : 1] = {};
  if (kVec) {
#pragma unroll
    for (int i = 0; i < 8; ++i) sa[kVec ? i : 0] = out.row_scale(ts, row0, i);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) out.store_rows(acc[i], i, sa[kVec ? i : 0]);
}

// The per-tensor form, for kernels that have no other.
template <bool kBf16Out>
__device__ __forceinline__ void store_wave_block(float4v (&acc)[8][8], const TensorScales ts, void* __restrict__ Dv, int64_t ldd,
                                                 bool accumulate, int64_t row0, int64_t col0, int rows, int cols, int lane) {
  store_wave_block_impl<kBf16Out, false>(acc, ts, Dv, ldd, accumulate, row0, col0, rows, cols, lane);
}

}  // namespace nvfp4
