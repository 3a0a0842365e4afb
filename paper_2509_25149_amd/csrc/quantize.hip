// NVFP4 quantizer kernels for gfx950 (App. B Eq. 1-4; Sec. 4.2-4.4; App. C).
//
// Work decomposition shared by both passes: a lane owns a 16-row x 8-column
// patch of the bf16 tensor (sixteen 128-bit loads, one per row); a wavefront
// owns 16 rows x 512 columns, so each of its loads reads 1 KiB of contiguous
// memory; a 256-thread workgroup covers 128 rows x 512 columns (four wavefronts,
// two 16-row groups each).  With this patch
//   - a 1x16 block of the row copy is split over two neighbouring lanes
//     (one cross-lane exchange of the half-block amax),
//   - a 1x16 block of the col copy (16 consecutive rows of one column) sits
//     entirely in one lane's registers, so the Hadamard butterfly and the
//     block amax need no cross-lane traffic,
//   - a 16x16 weight tile is exactly two neighbouring lanes,
//   - the eight columns of one row are the eight elements served by one
//     Philox call, whose output is shared by the row and the col copy.
// Row codes leave as one dword per lane and row (256 contiguous bytes per
// wavefront).  The transposed col copy, its scales and the row scales are staged
// in LDS and written back as contiguous 128-bit / 64-bit pieces: 64 bytes of
// codes per column per workgroup instead of scattered 8-byte stores.
#include "nvfp4_internal.h"
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

// unnormalised 16-point Walsh-Hadamard butterfly, stages h = 1, 2, 4, 8 (App. C)
__device__ __forceinline__ void butterfly16(float v[16]) {
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
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t m) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = max(m, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m), off, 64)));
  return m;
}

// ---------------------------------------------------------------- pass 1: amax (App. B.1)
// Every workgroup writes its own maxima (raw tensor / rotated tensor) into its
// slot of the workspace; a one-workgroup kernel folds the slots.  No atomics:
// thousands of same-address atomics serialise in L2 and cost more than the pass.
template <bool kRaw, bool kRht>
__global__ __launch_bounds__(kThreads) void amax_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                        int64_t cols, int64_t ld, uint32_t sign_mask,
                                                        uint32_t* __restrict__ ws) {
  __shared__ uint32_t red[2][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t col0 = static_cast<int64_t>(blockIdx.x) * kWaveCols + lane * 8;
  uint32_t m_raw = 0, m_rot = 0;
  float f_rot = 0.0f;
#pragma unroll 1
  for (int gi = 0; gi < kGroupsPerWave; ++gi) {
    const int64_t group = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock + wave * kGroupsPerWave + gi;
    if (col0 < cols && group * 16 < rows) {
      Patch p;
      load_patch(x, ld, group * 16, col0, p);
      if (kRaw) m_raw = max(m_raw, patch_amax_bits(p));
      if (kRht) {
        // The 1/4 normalisation is applied once to the maximum: rounding is monotone, so
        // max_i fl(0.25 v_i) = fl(0.25 max_i v_i).
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          float lo[16], hi[16];
          signed_column_pair(p, t, sign_mask, lo, hi);
          butterfly16(lo);
          butterfly16(hi);
#pragma unroll
          for (int r = 0; r < 16; ++r) f_rot = fmaxf(fmaxf(f_rot, fabsf(lo[r])), fabsf(hi[r]));
        }
      }
    }
  }
  if (kRaw) m_raw = wave_max_u32(m_raw);
  if (kRht) m_rot = wave_max_u32(__float_as_uint(0.25f * f_rot));
  if (lane == 0) {
    red[0][wave] = m_raw;
    red[1][wave] = m_rot;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t nwg = gridDim.x * gridDim.y, wg = blockIdx.y * gridDim.x + blockIdx.x;
    ws[kWsHeader + wg] = max(max(red[0][0], red[0][1]), max(red[0][2], red[0][3]));
    ws[kWsHeader + nwg + wg] = max(max(red[1][0], red[1][1]), max(red[1][2], red[1][3]));
  }
}

__global__ __launch_bounds__(1024) void amax_finalize_kernel(uint32_t* __restrict__ ws, uint32_t nwg) {
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
    uint32_t m = 0;
    for (int i = 0; i < 16; ++i) m = max(m, red[threadIdx.x][i]);
    ws[threadIdx.x] = m;
  }
}

// ---------------------------------------------------------------- pass 2: cast

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
    const uint32_t e = merge_bytes(cvt_sr_single<0>(v[0], rnd[0] << 16), cvt_sr_single<1>(v[2], rnd[1] << 16),
                                   cvt_sr_single<2>(v[4], rnd[2] << 16), cvt_sr_single<3>(v[6], rnd[3] << 16));
    const uint32_t o = merge_bytes(cvt_sr_single<0>(v[1], rnd[0] & 0xFFFF0000u), cvt_sr_single<1>(v[3], rnd[1] & 0xFFFF0000u),
                                   cvt_sr_single<2>(v[5], rnd[2] & 0xFFFF0000u), cvt_sr_single<3>(v[7], rnd[3] & 0xFFFF0000u));
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
    const uint32_t e = merge_bytes(cvt_sr_single<0>(v[0], draw_hi16(rnd, r0 + 0, c)), cvt_sr_single<1>(v[2], draw_hi16(rnd, r0 + 2, c)),
                                   cvt_sr_single<2>(v[4], draw_hi16(rnd, r0 + 4, c)), cvt_sr_single<3>(v[6], draw_hi16(rnd, r0 + 6, c)));
    const uint32_t o = merge_bytes(cvt_sr_single<0>(v[1], draw_hi16(rnd, r0 + 1, c)), cvt_sr_single<1>(v[3], draw_hi16(rnd, r0 + 3, c)),
                                   cvt_sr_single<2>(v[5], draw_hi16(rnd, r0 + 5, c)), cvt_sr_single<3>(v[7], draw_hi16(rnd, r0 + 7, c)));
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

template <bool kRow, bool kCol, bool kRht, bool kSR, bool k2D>
__global__ __launch_bounds__(kThreads, 2) void cast_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ld,
    const uint32_t* __restrict__ ws, uint32_t sign_mask, uint32_t key0, uint32_t key1,
    uint8_t* __restrict__ row_codes, uint8_t* __restrict__ row_scales, float* __restrict__ row_ts,
    uint8_t* __restrict__ col_codes, uint8_t* __restrict__ col_scales, float* __restrict__ col_ts) {
  __shared__ __attribute__((aligned(16))) uint8_t st_col_codes[kCol ? kColCodesBytes : 16];
  __shared__ __attribute__((aligned(16))) uint8_t st_col_scales[kCol ? kColScalesBytes : 16];
  __shared__ __attribute__((aligned(16))) uint8_t st_row_scales[kRow ? kRowScalesBytes : 16];
  __shared__ float lut_row[128], lut_col[128];  // block encode scale per stored E4M3 code

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t colblk = static_cast<int64_t>(blockIdx.x) * kWaveCols;
  const int64_t col0 = colblk + lane * 8;
  const int64_t group0 = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock;
  const int64_t ngroups = rows / 16;

  // App. B.1 Eq. 1, from the amax of pass 1.
  const float amax_raw = __uint_as_float(ws[0]);
  const float amax_col = kRht ? __uint_as_float(ws[1]) : amax_raw;
  float s_enc_r, s_dec_r, s_enc_c, s_dec_c;
  tensor_scales(amax_raw, s_enc_r, s_dec_r);
  tensor_scales(amax_col, s_enc_c, s_dec_c);
  if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) {
    if (kRow) { row_ts[0] = s_dec_r; row_ts[1] = amax_raw; }
    if (kCol) { col_ts[0] = s_dec_c; col_ts[1] = amax_col; }
  }
  // "real" block encode scale 1 / (fp32(code) * s_dec) for each of the 127 codes (App. B.2)
  {
    const int code = tid & 127;
    const float den = e4m3_decode(code) * (tid < 128 ? s_dec_r : s_dec_c);
    const float inv = (den == 0.0f || code == 127) ? 0.0f : 1.0f / den;
    if (tid < 128) lut_row[code] = inv; else lut_col[code] = inv;
  }
  __syncthreads();

#pragma unroll 1
  for (int gi = 0; gi < kGroupsPerWave; ++gi) {
    const int gl = wave * kGroupsPerWave + gi;  // group index inside the tile
    const int64_t group = group0 + gl;
    if (col0 >= cols || group >= ngroups) continue;
    const int64_t row0 = group * 16;

    Patch p;
    load_patch(x, ld, row0, col0, p);

    // Random words: one Philox call per row serves the row's 8 columns.
    uint32_t rnd[16][4];
    if (kSR) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        philox4x32_10(static_cast<uint32_t>(col0 >> 3), static_cast<uint32_t>(row0 + r), 0u, 0u, key0, key1, rnd[r]);
    }

    // 16x16 tile amax (Sec. 4.3): this lane's 16x8 half and the neighbour's.
    float s_enc_tile = 0.0f;
    uint32_t tile_code = 0;
    if (k2D) {
      uint32_t m = patch_amax_bits(p);
      m = max(m, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m), 1, 64)));
      tile_code = e4m3_encode(div_by_6(__uint_as_float(m)) * s_enc_r);   // Eq. 2-3
      s_enc_tile = lut_row[tile_code];
    }

    if (kRow) {
      const int64_t code_ld = cols / 2;
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
          m = fmaxf(m, __shfl_xor(m, 1, 64));
          code = e4m3_encode(div_by_6(m) * s_enc_r);                        // Eq. 2-3
          s_enc_b = lut_row[code];
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] *= s_enc_b;                    // Eq. 4
        const uint32_t d = encode8<kSR>(v, rnd[r]);
        *reinterpret_cast<uint32_t*>(row_codes + (row0 + r) * code_ld + col0 / 2) = d;
        if ((lane & 1) == 0) st_row_scales[(gl * 16 + r) * 32 + (lane >> 1)] = static_cast<uint8_t>(code);
      }
    }

    if (kCol) {
      auto emit_column = [&](float (&v)[16], int c) {
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
      };
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float lo[16], hi[16];
        signed_column_pair(p, t, kRht ? sign_mask : 0u, lo, hi);
        if (kRht) {
          butterfly16(lo);
          butterfly16(hi);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            lo[r] *= 0.25f;
            hi[r] *= 0.25f;
          }
        }
        emit_column(lo, 2 * t);
        emit_column(hi, 2 * t + 1);
      }
    }
  }
  __syncthreads();

  // ---- write-back of the staged pieces with wide, contiguous stores
  const int tile_groups = static_cast<int>(min<int64_t>(kGroupsPerBlock, ngroups - group0));
  const int tile_cols = static_cast<int>(min<int64_t>(kWaveCols, cols - colblk));

  if (kRow) {
    const int64_t scale_ld = cols / 16;
    const int nblk = tile_cols / 16;  // scale bytes per row in this tile
    if ((scale_ld & 15) == 0 && nblk == 32) {
      const int r = tid >> 1, half = tid & 1;   // 128 rows x two 16-byte halves
      if (r < tile_groups * 16)
        *reinterpret_cast<uint4*>(row_scales + (group0 * 16 + r) * scale_ld + colblk / 16 + half * 16) =
            *reinterpret_cast<const uint4*>(st_row_scales + r * 32 + half * 16);
    } else {
      for (int i = tid; i < tile_groups * 16 * nblk; i += kThreads) {
        const int r = i / nblk, b = i - r * nblk;
        row_scales[(group0 * 16 + r) * scale_ld + colblk / 16 + b] = st_row_scales[r * 32 + b];
      }
    }
  }

  if (kCol) {
    const int64_t code_ld = rows / 2, scale_ld = rows / 16;
    const bool wide = (code_ld & 15) == 0;   // 16-byte aligned column rows
#pragma unroll 1
    for (int i = 0; i < 8; ++i) {
      const int q = i * kThreads + tid;       // 2048 pieces of 16 bytes: column j, group pair pr
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
    for (int i = 0; i < 2; ++i) {
      const int j = i * kThreads + tid;       // one column: 8 scale bytes (one per group)
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

// ---------------------------------------------------------------- host side

size_t quantize_workspace_bytes(int64_t rows, int64_t cols) {
  const int64_t gx = (cols + kWaveCols - 1) / kWaveCols, gy = (rows / 16 + kGroupsPerBlock - 1) / kGroupsPerBlock;
  return static_cast<size_t>(kWsHeader + 2 * gx * gy) * sizeof(uint32_t);
}

template <bool kRow, bool kCol, bool kRht, bool kSR, bool k2D>
static void launch_cast(const QuantizeArgs& a, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL((cast_kernel<kRow, kCol, kRht, kSR, k2D>), grid, dim3(kThreads), 0, s,
                     static_cast<const uint16_t*>(a.x), a.rows, a.cols, a.ld, a.ws, a.sign_mask, a.key0,
                     a.key1, a.row_codes, a.row_scales, a.row_ts, a.col_codes, a.col_scales, a.col_ts);
}

template <bool kRow, bool kCol, bool kRht>
static void dispatch_cast2(const QuantizeArgs& a, dim3 grid, hipStream_t s) {
  if (a.block2d) {
    if (a.sr) launch_cast<kRow, kCol, false, true, true>(a, grid, s);
    else launch_cast<kRow, kCol, false, false, true>(a, grid, s);
  } else {
    if (a.sr) launch_cast<kRow, kCol, kRht, true, false>(a, grid, s);
    else launch_cast<kRow, kCol, kRht, false, false>(a, grid, s);
  }
}

hipError_t launch_quantize(const QuantizeArgs& a, hipStream_t s) {
  const dim3 grid(static_cast<unsigned>((a.cols + kWaveCols - 1) / kWaveCols),
                  static_cast<unsigned>((a.rows / 16 + kGroupsPerBlock - 1) / kGroupsPerBlock));
  const bool rht = a.want_col && a.rht;
  const bool raw = a.want_row || !rht;
  const uint16_t* x = static_cast<const uint16_t*>(a.x);
  if (raw && rht)
    hipLaunchKernelGGL((amax_kernel<true, true>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.sign_mask, a.ws);
  else if (rht)
    hipLaunchKernelGGL((amax_kernel<false, true>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.sign_mask, a.ws);
  else
    hipLaunchKernelGGL((amax_kernel<true, false>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.sign_mask, a.ws);
  hipLaunchKernelGGL(amax_finalize_kernel, dim3(1), dim3(1024), 0, s, a.ws, grid.x * grid.y);
  if (a.want_row && a.want_col) {
    if (rht) dispatch_cast2<true, true, true>(a, grid, s);
    else dispatch_cast2<true, true, false>(a, grid, s);
  } else if (a.want_row) {
    dispatch_cast2<true, false, false>(a, grid, s);
  } else {
    if (rht) dispatch_cast2<false, true, true>(a, grid, s);
    else dispatch_cast2<false, true, false>(a, grid, s);
  }
  return hipGetLastError();
}

}  // namespace nvfp4
