// Pieces shared by the NVFP4 quantizer kernels for gfx950: the 16-row x 8-column patch a lane owns,
// the code packing of App. B.3 (Eq. 4) for both rounding modes, the LDS staging of one 128-row x
// 512-column workgroup tile and its write-back.  Device code only.
#pragma once

#include "nvfp4_device.h"

namespace nvfp4 {

constexpr int kThreads = 256;
constexpr int kWaveCols = 512;      // 64 lanes x 8 columns
constexpr int kGroupsPerWave = 2;   // 16-row groups a wavefront walks through
constexpr int kGroupsPerBlock = 8;  // 4 wavefronts x 2 groups = 128 rows per workgroup
constexpr int kWsHeader = 16;       // words before the per-workgroup partial maxima

struct Patch {
  uint4 raw[16];  // raw[r] = 8 bf16 of row r, columns col0..col0+7
};

__device__ __forceinline__ float patch_elem(const uint4& q, int c) {
  const uint32_t w = (c < 2) ? q.x : (c < 4) ? q.y : (c < 6) ? q.z : q.w;
  return (c & 1) ? bf16_hi(w) : bf16_lo(w);
}

__device__ __forceinline__ void load_patch(const uint16_t* __restrict__ x, int64_t ld, int64_t row0,
                                           int64_t col0, Patch& p) {
#pragma unroll
  for (int r = 0; r < 16; ++r)
    p.raw[r] = *reinterpret_cast<const uint4*>(x + (row0 + r) * ld + col0);
}

typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));

// max |bf16| of a patch, as FP32 bits (also carries Inf/NaN through as the largest
// pattern): magnitudes of bf16 order like 15-bit integers, two per dword (v_pk_max_u16).
__device__ __forceinline__ uint32_t patch_amax_bits(const Patch& p) {
  union U {
    uint32_t u;
    ushort2v v;
  };
  U m;
  m.u = 0u;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const uint32_t w[4] = {p.raw[r].x, p.raw[r].y, p.raw[r].z, p.raw[r].w};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      U a;
      a.u = w[t] & 0x7FFF7FFFu;
      m.v = __builtin_elementwise_max(m.v, a.v);
    }
  }
  return max(m.u & 0xFFFFu, m.u >> 16) << 16;
}

// The 16 values of column pair t (columns 2t, 2t+1) of a patch, sign diagonal applied:
// lo[r], hi[r] = +-x[row r][2t], +-x[row r][2t+1] as FP32.  The sign of row r is the same for
// every column, so it is one XOR on the packed bf16 word.
__device__ __forceinline__ void signed_column_pair(const Patch& p, int t, uint32_t sign_mask, float lo[16], float hi[16]) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const uint32_t w = (t == 0 ? p.raw[r].x : t == 1 ? p.raw[r].y : t == 2 ? p.raw[r].z : p.raw[r].w) ^
                       (((sign_mask >> r) & 1u) * 0x80008000u);
    lo[r] = bf16_lo(w);
    hi[r] = bf16_hi(w);
  }
}

// Unnormalised Walsh-Hadamard butterfly over the 16 rows a lane holds, stages h = 1, 2, ... < kStagesBelow
// (App. C).  kStagesBelow = 16 is the whole 16-point transform; 2 and 4 rotate every aligned pair / group of
// four on its own; the first four stages of a 32- or 128-point transform are the 16-point one.
template <int kStagesBelow>
__device__ __forceinline__ void butterfly_rows(float v[16]) {
#pragma unroll
  for (int h = 1; h < kStagesBelow; h <<= 1) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if ((i & h) == 0) {
        const float a = v[i], b = v[i + h];
        v[i] = a + b;
        v[i + h] = a - b;
      }
    }
  }
}

// binary32 nearest to 1 / sqrt(d), the normalisation of the d-point rotation (exact for d = 4, 16)
template <int kD>
__device__ __forceinline__ constexpr float rht_norm() {
  return kD == 2 ? 0.707106781186547524f : kD == 4 ? 0.5f : kD == 16 ? 0.25f : kD == 32 ? 0.176776695296636893f
                                                                                        : 0.0883883476483184405f;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t m) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = max(m, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m), off, 64)));
  return m;
}

// Eight scaled values of one row -> one dword of eight codes.
template <bool kSR>
__device__ __forceinline__ uint32_t encode8(const float v[8], const uint32_t rnd[4]) {
  if (!kSR) {
    uint32_t d = 0;
    d = cvt_rne_pair<0>(d, v[0], v[1]);
    d = cvt_rne_pair<1>(d, v[2], v[3]);
    d = cvt_rne_pair<2>(d, v[4], v[5]);
    d = cvt_rne_pair<3>(d, v[6], v[7]);
    return d;
  } else {
    uint32_t e = 0u, o = 0u;   // low nibble of byte t: element 2t (e) / 2t + 1 (o)
    cvt_sr_single_into<0>(e, v[0], rnd[0] << 16);
    cvt_sr_single_into<1>(e, v[2], rnd[1] << 16);
    cvt_sr_single_into<2>(e, v[4], rnd[2] << 16);
    cvt_sr_single_into<3>(e, v[6], rnd[3] << 16);
    cvt_sr_single_into<0>(o, v[1], rnd[0] & 0xFFFF0000u);
    cvt_sr_single_into<1>(o, v[3], rnd[1] & 0xFFFF0000u);
    cvt_sr_single_into<2>(o, v[5], rnd[2] & 0xFFFF0000u);
    cvt_sr_single_into<3>(o, v[7], rnd[3] & 0xFFFF0000u);
    return interleave_nibbles(e, o);
  }
}

// The 16-bit draw of element (row r of the patch, column c of the patch),
// moved to the top half of a word.
__device__ __forceinline__ uint32_t draw_hi16(const uint32_t rnd[16][4], int r, int c) {
  const uint32_t w = rnd[r][c >> 1];
  return (c & 1) ? (w & 0xFFFF0000u) : (w << 16);
}

// Eight scaled values of one column (rows r0..r0+7 of the patch) -> one dword.
template <bool kSR>
__device__ __forceinline__ uint32_t encode8_col(const float* v, const uint32_t rnd[16][4], int r0, int c) {
  if (!kSR) {
    const uint32_t none[4] = {0, 0, 0, 0};
    return encode8<false>(v, none);
  } else {
    uint32_t e = 0u, o = 0u;
    cvt_sr_single_into<0>(e, v[0], draw_hi16(rnd, r0 + 0, c));
    cvt_sr_single_into<1>(e, v[2], draw_hi16(rnd, r0 + 2, c));
    cvt_sr_single_into<2>(e, v[4], draw_hi16(rnd, r0 + 4, c));
    cvt_sr_single_into<3>(e, v[6], draw_hi16(rnd, r0 + 6, c));
    cvt_sr_single_into<0>(o, v[1], draw_hi16(rnd, r0 + 1, c));
    cvt_sr_single_into<1>(o, v[3], draw_hi16(rnd, r0 + 3, c));
    cvt_sr_single_into<2>(o, v[5], draw_hi16(rnd, r0 + 5, c));
    cvt_sr_single_into<3>(o, v[7], draw_hi16(rnd, r0 + 7, c));
    return interleave_nibbles(e, o);
  }
}

// LDS staging of one workgroup tile (128 rows x 512 columns):
//   col codes : [c 0..7][g 0..7][65 slots of 8 B]  (lane l of group g, column c of its patch)
//               -- consecutive lanes write consecutive slots; the 65th slot is padding that
//               spreads the transposed read-back over the banks
//   col scales: [c][g][64] bytes ; row scales: [128 rows][32] bytes
constexpr int kColSlot = 65;
constexpr int kColCodesBytes = 8 * kGroupsPerBlock * kColSlot * 8;   // 33280
constexpr int kColScalesBytes = 8 * kGroupsPerBlock * 64;            // 4096
constexpr int kRowScalesBytes = 16 * kGroupsPerBlock * 32;           // 4096

// Folds the per-workgroup maxima of pass 1 (nwg raw maxima, then nwg rotated maxima, after the header):
// ws[0] = amax of the tensor, ws[1] = amax of the rotated tensor, both as FP32 bits (also stored to `copy` if
// given).  One workgroup of 1024.
static __global__ __launch_bounds__(1024) void amax_finalize_kernel(uint32_t* __restrict__ ws, uint32_t nwg,
                                                                   uint32_t* __restrict__ copy) {
  __shared__ uint32_t red[2][16];
  uint32_t m0 = 0, m1 = 0;
  for (uint32_t i = threadIdx.x; i < nwg; i += 1024) {
    m0 = max(m0, ws[kWsHeader + i]);
    m1 = max(m1, ws[kWsHeader + nwg + i]);
  }
  m0 = wave_max_u32(m0);
  m1 = wave_max_u32(m1);
  if ((threadIdx.x & 63) == 0) {
    red[0][threadIdx.x >> 6] = m0;
    red[1][threadIdx.x >> 6] = m1;
  }
  __syncthreads();
  if (threadIdx.x < 2) {
    uint32_t m = 0, raw = 0;
    for (int i = 0; i < 16; ++i) {
      m = max(m, red[threadIdx.x][i]);
      raw = max(raw, red[0][i]);
    }
    // a non-finite input shows in the rotated amax too (the maxima of rotated values skip NaNs)
    if (raw >= 0x7F800000u) m = max(m, raw);
    ws[threadIdx.x] = m;
    if (copy) copy[threadIdx.x] = m;
  }
}

// Row copy of one patch (App. B.2-B.3): per row, the amax of the 1x16 block (this lane's eight columns and the
// neighbour's; or the 16x16 tile's scale of Sec. 4.3), Eq. 2-4, one dword of codes straight to memory (dst = the
// row copy's codes at (first row of the patch, first column of the lane)), the scale byte staged in LDS.
template <bool kSR, bool k2D>
__device__ __forceinline__ void row_pass(const Patch& p, const uint32_t (&rnd)[16][4], int lane, int gl, float s_enc_r,
                                         const float* lut_row, float s_enc_tile, uint32_t tile_code,
                                         uint8_t* __restrict__ dst, int64_t code_ld, uint8_t* st_row_scales) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float v[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = patch_elem(p.raw[r], c);
    float s_enc_b;
    uint32_t code;
    if (k2D) {
      s_enc_b = s_enc_tile;
      code = tile_code;
    } else {
      float m = 0.0f;
#pragma unroll
      for (int c = 0; c < 8; ++c) m = fmaxf(m, fabsf(v[c]));
      m = fmaxf(m, lane_xor1(m));
      code = e4m3_encode(div_by_6(m) * s_enc_r);                        // Eq. 2-3
      s_enc_b = lut_row[code];
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] *= s_enc_b;                    // Eq. 4
    const uint32_t d = encode8<kSR>(v, rnd[r]);
    *reinterpret_cast<uint32_t*>(dst + r * code_ld) = d;
    if ((lane & 1) == 0) st_row_scales[(gl * 16 + r) * 32 + (lane >> 1)] = static_cast<uint8_t>(code);
  }
}

// One 1x16 block of the col copy: the 16 (possibly rotated) values of column c of the patch -> scale byte and
// eight bytes of codes, staged in LDS.
template <bool kSR, bool k2D>
__device__ __forceinline__ void emit_column(float (&v)[16], int c, const uint32_t (&rnd)[16][4], int lane, int gl,
                                            float s_enc_c, const float* lut_col, float s_enc_tile, uint32_t tile_code,
                                            uint8_t* st_col_codes, uint8_t* st_col_scales) {
  float s_enc_b;
  uint32_t code;
  if (k2D) {
    s_enc_b = s_enc_tile;
    code = tile_code;
  } else {
    float m = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) m = fmaxf(fmaxf(m, fabsf(v[r])), fabsf(v[r + 1]));
    code = e4m3_encode(div_by_6(m) * s_enc_c);
    s_enc_b = lut_col[code];
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] *= s_enc_b;
  uint2 out;
  out.x = encode8_col<kSR>(v, rnd, 0, c);
  out.y = encode8_col<kSR>(v + 8, rnd, 8, c);
  *reinterpret_cast<uint2*>(st_col_codes + ((c * kGroupsPerBlock + gl) * kColSlot + lane) * 8) = out;
  st_col_scales[(c * kGroupsPerBlock + gl) * 64 + lane] = static_cast<uint8_t>(code);
}

// Write-back of one staged workgroup tile with wide, contiguous stores (all kT threads of the workgroup call it
// after a barrier that follows the last staging write).
template <bool kRow, bool kCol, int kT>
__device__ __forceinline__ void write_back_tile(int tid, int64_t rows, int64_t cols, int64_t group0, int64_t ngroups,
                                                int64_t colblk, const uint8_t* st_col_codes, const uint8_t* st_col_scales,
                                                const uint8_t* st_row_scales, uint8_t* __restrict__ row_scales,
                                                uint8_t* __restrict__ col_codes, uint8_t* __restrict__ col_scales) {
  const int tile_groups = static_cast<int>(min<int64_t>(kGroupsPerBlock, ngroups - group0));
  const int tile_cols = static_cast<int>(min<int64_t>(kWaveCols, cols - colblk));

  if (kRow) {
    const int64_t scale_ld = cols / 16;
    const int nblk = tile_cols / 16;  // scale bytes per row in this tile
    if ((scale_ld & 15) == 0 && nblk == 32) {
      for (int q = tid; q < 256; q += kT) {
        const int r = q >> 1, half = q & 1;   // 128 rows x two 16-byte halves
        if (r < tile_groups * 16)
          *reinterpret_cast<uint4*>(row_scales + (group0 * 16 + r) * scale_ld + colblk / 16 + half * 16) =
              *reinterpret_cast<const uint4*>(st_row_scales + r * 32 + half * 16);
      }
    } else {
      for (int i = tid; i < tile_groups * 16 * nblk; i += kT) {
        const int r = i / nblk, b = i - r * nblk;
        row_scales[(group0 * 16 + r) * scale_ld + colblk / 16 + b] = st_row_scales[r * 32 + b];
      }
    }
  }

  if (kCol) {
    const int64_t code_ld = rows / 2, scale_ld = rows / 16;
    const bool wide = (code_ld & 15) == 0;   // 16-byte aligned column rows
#pragma unroll 1
    for (int i = 0; i < 2048 / kT; ++i) {
      const int q = i * kT + tid;       // 2048 pieces of 16 bytes: column j, group pair pr
      const int j = q >> 2, pr = q & 3;
      if (j >= tile_cols) continue;
      const int lj = j >> 3, c = j & 7;
      const uint2 a = *reinterpret_cast<const uint2*>(st_col_codes + ((c * kGroupsPerBlock + 2 * pr) * kColSlot + lj) * 8);
      const uint2 b = *reinterpret_cast<const uint2*>(st_col_codes + ((c * kGroupsPerBlock + 2 * pr + 1) * kColSlot + lj) * 8);
      uint8_t* dst = col_codes + (colblk + j) * code_ld + (group0 + 2 * pr) * 8;
      if (wide && 2 * pr + 1 < tile_groups) {
        *reinterpret_cast<uint4*>(dst) = make_uint4(a.x, a.y, b.x, b.y);
      } else {
        if (2 * pr < tile_groups) *reinterpret_cast<uint2*>(dst) = a;
        if (2 * pr + 1 < tile_groups) *reinterpret_cast<uint2*>(dst + 8) = b;
      }
    }
#pragma unroll 1
    for (int i = 0; i < 512 / kT; ++i) {
      const int j = i * kT + tid;       // one column: 8 scale bytes (one per group)
      if (j >= tile_cols) continue;
      const int lj = j >> 3, c = j & 7;
      uint8_t sc[8];
#pragma unroll
      for (int g = 0; g < 8; ++g) sc[g] = st_col_scales[(c * kGroupsPerBlock + g) * 64 + lj];
      uint8_t* dst = col_scales + (colblk + j) * scale_ld + group0;
      if (tile_groups == 8 && (scale_ld & 7) == 0) {
        uint2 o;
        o.x = sc[0] | (sc[1] << 8) | (sc[2] << 16) | (static_cast<uint32_t>(sc[3]) << 24);
        o.y = sc[4] | (sc[5] << 8) | (sc[6] << 16) | (static_cast<uint32_t>(sc[7]) << 24);
        *reinterpret_cast<uint2*>(dst) = o;
      } else {
        for (int g = 0; g < tile_groups; ++g) dst[g] = sc[g];
      }
    }
  }
}

}  // namespace nvfp4
