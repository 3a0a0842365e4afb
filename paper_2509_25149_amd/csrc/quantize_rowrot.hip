// NVFP4 quantizer with the row copy rotated as well (gfx950): the 16-point random Hadamard transform applied to the
// operands of Fprop and Dgrad, the variant Sec. 4.2 leaves out of the recipe and App. E.4.1 ablates.  The row copy's
// contraction dimension is the tensor's columns, so every aligned group of 16 consecutive columns of a row is
// multiplied by the sign diagonal and H_16 before scaling (App. C), with the same seed as the col copy's rotation.
//
// Same work decomposition as the plain quantizer: a lane owns 16 rows x 8 columns, so a group of 16 columns is
// two neighbouring lanes.  Butterfly stages h = 1, 2, 4 run on the lane's own eight values of a row, stage h = 8
// takes the neighbour's value through a DPP lane swap (even lane: own + other, odd lane: other - own), then the
// multiply by 1/4: the stage order and every rounding are those of the in-lane transform of the col copy.
#include "nvfp4_internal.h"
#include "quantize_tile.h"

namespace nvfp4 {

namespace {

// XOR words that apply the sign diagonal to the four packed bf16 pairs of a lane's eight columns: the lane holds
// columns 0..7 (even lane) or 8..15 (odd lane) of its group of 16.
__device__ __forceinline__ void lane_sign_words(uint32_t sign_mask, int lane, uint32_t sgn[4]) {
  const uint32_t bits = (sign_mask >> ((lane & 1) * 8)) & 0xFFu;
#pragma unroll
  for (int t = 0; t < 4; ++t) sgn[t] = (((bits >> (2 * t)) & 1u) << 15) | (((bits >> (2 * t + 1)) & 1u) << 31);
}

// The lane's eight values of row r after the 16-point rotation along the columns, not yet normalised.
__device__ __forceinline__ void rotated_row(const uint4& q, const uint32_t sgn[4], bool odd, float v[8]) {
  const uint32_t w[4] = {q.x ^ sgn[0], q.y ^ sgn[1], q.z ^ sgn[2], q.w ^ sgn[3]};
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    v[2 * t] = bf16_lo(w[t]);
    v[2 * t + 1] = bf16_hi(w[t]);
  }
#pragma unroll
  for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if ((i & h) == 0) {
        const float a = v[i], b = v[i + h];
        v[i] = a + b;
        v[i + h] = a - b;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float o = lane_xor1(v[i]);
    v[i] = odd ? o - v[i] : v[i] + o;
  }
}

// ---------------------------------------------------------------- pass 1: amax (App. B.1) of up to three spaces
// ws slots per workgroup: raw maxima, col-rotated maxima, row-rotated maxima (three runs of nwg words).
template <int kColRht>   // kColRht: 0 or 16
__global__ __launch_bounds__(kThreads) void amax_rowrot_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                               int64_t ld, uint32_t sign_mask, uint32_t* __restrict__ ws) {
  __shared__ uint32_t red[3][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t col0 = static_cast<int64_t>(blockIdx.x) * kWaveCols + lane * 8;
  uint32_t sgn[4];
  lane_sign_words(sign_mask, lane, sgn);
  uint32_t m_raw = 0;
  float f_col = 0.0f, f_row = 0.0f;
#pragma unroll 1
  for (int gi = 0; gi < kGroupsPerWave; ++gi) {
    const int64_t group = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock + wave * kGroupsPerWave + gi;
    // cols is a multiple of 16, so both lanes of a pair are inside or outside together
    if (col0 < cols && group * 16 < rows) {
      Patch p;
      load_patch(x, ld, group * 16, col0, p);
      m_raw = max(m_raw, patch_amax_bits(p));   // always: a NaN in the input shows here only
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v[8];
        rotated_row(p.raw[r], sgn, lane & 1, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) f_row = fmaxf(f_row, fabsf(v[i]));
      }
      if (kColRht) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          float lo[16], hi[16];
          signed_column_pair(p, t, sign_mask, lo, hi);
          butterfly_rows<kColRht>(lo);
          butterfly_rows<kColRht>(hi);
#pragma unroll
          for (int r = 0; r < 16; ++r) f_col = fmaxf(fmaxf(f_col, fabsf(lo[r])), fabsf(hi[r]));
        }
      }
    }
  }
  // the normalisation is applied once to each maximum (rounding is monotone; 1/4 is exact anyway)
  m_raw = wave_max_u32(m_raw);
  const uint32_t m_col = wave_max_u32(__float_as_uint(0.25f * f_col));
  const uint32_t m_row = wave_max_u32(__float_as_uint(0.25f * f_row));
  if (lane == 0) {
    red[0][wave] = m_raw;
    red[1][wave] = m_col;
    red[2][wave] = m_row;
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    const uint32_t nwg = gridDim.x * gridDim.y, wg = blockIdx.y * gridDim.x + blockIdx.x;
    const int k = threadIdx.x;
    ws[kWsHeader + k * nwg + wg] = max(max(red[k][0], red[k][1]), max(red[k][2], red[k][3]));
  }
}

// Folds the three runs of per-workgroup maxima: ws[0] raw, ws[1] col-rotated, ws[2] row-rotated amax (FP32 bits).
__global__ __launch_bounds__(1024) void amax_finalize3_kernel(uint32_t* __restrict__ ws, uint32_t nwg) {
  __shared__ uint32_t red[3][16];
  uint32_t m[3] = {0, 0, 0};
  for (uint32_t i = threadIdx.x; i < nwg; i += 1024) {
#pragma unroll
    for (int k = 0; k < 3; ++k) m[k] = max(m[k], ws[kWsHeader + k * nwg + i]);
  }
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    m[k] = wave_max_u32(m[k]);
    if ((threadIdx.x & 63) == 0) red[k][threadIdx.x >> 6] = m[k];
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    uint32_t f = 0, raw = 0;
    for (int i = 0; i < 16; ++i) {
      f = max(f, red[threadIdx.x][i]);
      raw = max(raw, red[0][i]);
    }
    // a non-finite input shows in every copy's amax (the maxima of rotated values skip NaNs)
    if (raw >= 0x7F800000u) f = max(f, raw);
    ws[threadIdx.x] = f;
  }
}

// ---------------------------------------------------------------- pass 2: cast
// Row copy of one patch, rotated along the columns (App. C), then App. B.2-B.3 as in the plain row pass.
template <bool kSR>
__device__ __forceinline__ void row_pass_rotated(const Patch& p, const uint32_t (&rnd)[16][4], const uint32_t sgn[4], int lane,
                                                 int gl, float s_enc_r, const float* lut_row, uint8_t* __restrict__ dst,
                                                 int64_t code_ld, uint8_t* st_row_scales) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float v[8];
    rotated_row(p.raw[r], sgn, lane & 1, v);
    float m = 0.0f;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      v[c] *= 0.25f;
      m = fmaxf(m, fabsf(v[c]));
    }
    m = fmaxf(m, lane_xor1(m));
    const uint32_t code = e4m3_encode(div_by_6(m) * s_enc_r);          // Eq. 2-3
    const float s_enc_b = lut_row[code];
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] *= s_enc_b;                      // Eq. 4
    const uint32_t d = encode8<kSR>(v, rnd[r]);
    *reinterpret_cast<uint32_t*>(dst + r * code_ld) = d;
    if ((lane & 1) == 0) st_row_scales[(gl * 16 + r) * 32 + (lane >> 1)] = static_cast<uint8_t>(code);
  }
}

template <bool kCol, int kColRht, bool kSR>   // kColRht: 0 or 16
__global__ __launch_bounds__(kThreads, 2) void cast_rowrot_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ld, const uint32_t* __restrict__ ws,
    uint32_t sign_mask, uint32_t key0, uint32_t key1, uint8_t* __restrict__ row_codes, uint8_t* __restrict__ row_scales,
    float* __restrict__ row_ts, uint8_t* __restrict__ col_codes, uint8_t* __restrict__ col_scales, float* __restrict__ col_ts) {
  __shared__ __attribute__((aligned(16))) uint8_t st_col_codes[kCol ? kColCodesBytes : 16];
  __shared__ __attribute__((aligned(16))) uint8_t st_col_scales[kCol ? kColScalesBytes : 16];
  __shared__ __attribute__((aligned(16))) uint8_t st_row_scales[kRowScalesBytes];
  __shared__ float lut_row[128], lut_col[128];  // block encode scale per stored E4M3 code

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t colblk = static_cast<int64_t>(blockIdx.x) * kWaveCols;
  const int64_t col0 = colblk + lane * 8;
  const int64_t group0 = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock;
  const int64_t ngroups = rows / 16;

  // App. B.1 Eq. 1: each copy from the amax of the space it is quantized in.
  const float amax_row = __uint_as_float(ws[2]);
  const float amax_col = __uint_as_float(kColRht ? ws[1] : ws[0]);
  float s_enc_r, s_dec_r, s_enc_c, s_dec_c;
  tensor_scales(amax_row, s_enc_r, s_dec_r);
  tensor_scales(amax_col, s_enc_c, s_dec_c);
  if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) {
    row_ts[0] = s_dec_r;
    row_ts[1] = amax_row;
    if (kCol) { col_ts[0] = s_dec_c; col_ts[1] = amax_col; }
  }
  {
    const int code = tid & 127;
    const float den = e4m3_decode(code) * (tid < 128 ? s_dec_r : s_dec_c);
    const float inv = (den == 0.0f || code == 127) ? 0.0f : 1.0f / den;
    if (tid < 128) lut_row[code] = inv; else lut_col[code] = inv;
  }
  __syncthreads();

  uint32_t sgn[4];
  lane_sign_words(sign_mask, lane, sgn);
  // without a rotation of the col copy its values carry no signs
  const uint32_t col_sign_mask = kColRht ? sign_mask : 0u;

#pragma unroll 1
  for (int gi = 0; gi < kGroupsPerWave; ++gi) {
    const int gl = wave * kGroupsPerWave + gi;
    const int64_t group = group0 + gl;
    if (col0 >= cols || group >= ngroups) continue;   // pairs of lanes leave together (cols is a multiple of 16)
    const int64_t row0 = group * 16;

    Patch p;
    load_patch(x, ld, row0, col0, p);

    uint32_t rnd[16][4];
    if (kSR) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        philox4x32_10(static_cast<uint32_t>(col0 >> 3), static_cast<uint32_t>(row0 + r), 0u, 0u, key0, key1, rnd[r]);
    }

    row_pass_rotated<kSR>(p, rnd, sgn, lane, gl, s_enc_r, lut_row, row_codes + row0 * (cols / 2) + col0 / 2, cols / 2,
                          st_row_scales);

    if (kCol) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float lo[16], hi[16];
        signed_column_pair(p, t, col_sign_mask, lo, hi);
        if (kColRht) {
          butterfly_rows<kColRht>(lo);
          butterfly_rows<kColRht>(hi);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            lo[r] *= 0.25f;
            hi[r] *= 0.25f;
          }
        }
        emit_column<kSR, false>(lo, 2 * t, rnd, lane, gl, s_enc_c, lut_col, 0.0f, 0u, st_col_codes, st_col_scales);
        emit_column<kSR, false>(hi, 2 * t + 1, rnd, lane, gl, s_enc_c, lut_col, 0.0f, 0u, st_col_codes, st_col_scales);
      }
    }
  }
  __syncthreads();

  write_back_tile<true, kCol, kThreads>(tid, rows, cols, group0, ngroups, colblk, st_col_codes, st_col_scales, st_row_scales,
                                        row_scales, col_codes, col_scales);
}

template <bool kCol, int kColRht>
void launch_both(const QuantizeArgs& a, dim3 grid, hipStream_t s) {
  const uint16_t* x = static_cast<const uint16_t*>(a.x);
  hipLaunchKernelGGL((amax_rowrot_kernel<kColRht>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.sign_mask, a.ws);
  hipLaunchKernelGGL(amax_finalize3_kernel, dim3(1), dim3(1024), 0, s, a.ws, grid.x * grid.y);
  if (a.sr)
    hipLaunchKernelGGL((cast_rowrot_kernel<kCol, kColRht, true>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.ws,
                       a.sign_mask, a.key0, a.key1, a.row_codes, a.row_scales, a.row_ts, a.col_codes, a.col_scales, a.col_ts);
  else
    hipLaunchKernelGGL((cast_rowrot_kernel<kCol, kColRht, false>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.ws,
                       a.sign_mask, a.key0, a.key1, a.row_codes, a.row_scales, a.row_ts, a.col_codes, a.col_scales, a.col_ts);
}

}  // namespace

// a.row_rht is set: 1x16 blocks, both passes, a row copy, and a col copy that is absent, plain or rotated with d = 16.
hipError_t launch_quantize_rowrot(const QuantizeArgs& a, hipStream_t s) {
  const dim3 grid(static_cast<unsigned>((a.cols + kWaveCols - 1) / kWaveCols),
                  static_cast<unsigned>((a.rows / 16 + kGroupsPerBlock - 1) / kGroupsPerBlock));
  if (!a.want_col) launch_both<false, 0>(a, grid, s);
  else if (a.rht_dim == 16) launch_both<true, 16>(a, grid, s);
  else launch_both<true, 0>(a, grid, s);
  return hipGetLastError();
}

}  // namespace nvfp4
