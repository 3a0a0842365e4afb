// NVFP4 quantizer with a 32- or 128-point rotation of the col copy, for gfx950 (Sec. 4.2 "Hadamard matrix size"
// and App. E.4 ablate these sizes against the 16-point choice; construction of App. C).
//
// A rotation group of d = 16 G rows (G = 2 or 8) spans G of the 16-row groups that the 16-point kernels give to
// one lane each, so the d-point butterfly is split as H_d = H_G (x) H_16: stages h = 1..8 run in the lane's
// registers as before; stages h = 16.. combine the same (row-in-group, column) position of G different groups,
// which live in G different wavefronts.  A workgroup is therefore 8 wavefronts, wavefront w owning group w of the
// 128-row x 512-column tile (128 rows are whole rotation groups for both sizes), and the cross-group stages go
// through LDS one patch column at a time:
//   1. every wavefront stores its 16 values of the column      [group][row][lane]
//   2. wavefront w loads rows 2w, 2w+1 of all 8 groups, runs the remaining stages over the group index and stores
//      the results in place
//   3. every wavefront reads its own 16 values back, applies the 1/sqrt(d) factor and carries on exactly like the
//      16-point kernel (block amax, scale, codes; Eq. 2-4).
// The stage order and the single final multiply are the same as in a straight d-point butterfly, so results are
// bit-identical to it.  The row copy is never rotated and is produced in the same pass.
#include "nvfp4_internal.h"
#include "quantize_tile.h"

namespace nvfp4 {

namespace {

constexpr int kWideThreads = 512;

// Stages h = 16, 32, .. < 16 kG of the butterfly over the group index, for the two rows this wavefront serves.
// Groups at or beyond tile_groups hold nothing; they come in whole rotation groups, so skipping them whole is exact.
template <int kG, bool kStore>
__device__ __forceinline__ float cross_group_stages(float* xch, int wave, int lane, int tile_groups) {
  float m = 0.0f;
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    float* base = xch + (2 * wave + rr) * 64 + lane;
    float u[8];
#pragma unroll
    for (int g = 0; g < 8; ++g) u[g] = base[g * 16 * 64];
#pragma unroll
    for (int h = 1; h < kG; h <<= 1) {
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        if ((g & h) == 0) {
          const float a = u[g], b = u[g + h];
          u[g] = a + b;
          u[g + h] = a - b;
        }
      }
    }
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      if (kStore) base[g * 16 * 64] = u[g];
      else if (g < tile_groups) m = fmaxf(m, fabsf(u[g]));
    }
  }
  return m;
}

// The 16 sign bits of the rows of group `group` (rows 16 group .. 16 group + 15) inside their rotation group.
template <int kD>
__device__ __forceinline__ uint32_t group_signs(uint4 sign_words, int64_t group) {
  const int g = static_cast<int>(group & (kD / 16 - 1));
  const uint32_t w = (g >> 1) == 0 ? sign_words.x : (g >> 1) == 1 ? sign_words.y : (g >> 1) == 2 ? sign_words.z : sign_words.w;
  return (w >> ((g & 1) * 16)) & 0xFFFFu;
}

// ---------------------------------------------------------------- pass 1: amax (App. B.1), raw and rotated
template <int kD>
__global__ __launch_bounds__(kWideThreads) void amax_wide_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                                 int64_t ld, uint4 sign_words, uint32_t* __restrict__ ws) {
  __shared__ float xch[8 * 16 * 64];
  __shared__ uint32_t red[2][8];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t col0 = static_cast<int64_t>(blockIdx.x) * kWaveCols + lane * 8;
  const int64_t group0 = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock, group = group0 + wave;
  const int64_t ngroups = rows / 16;
  const int tile_groups = static_cast<int>(min<int64_t>(kGroupsPerBlock, ngroups - group0));
  const bool col_ok = col0 < cols, active = col_ok && group < ngroups;

  Patch p;
  if (active) {
    load_patch(x, ld, group * 16, col0, p);
  } else {
#pragma unroll
    for (int r = 0; r < 16; ++r) p.raw[r] = make_uint4(0u, 0u, 0u, 0u);
  }
  const uint32_t m_raw = wave_max_u32(patch_amax_bits(p));   // always: see amax_kernel

  const uint32_t signs = group_signs<kD>(sign_words, group);
  float f_rot = 0.0f;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    float lo[16], hi[16];
    signed_column_pair(p, t, signs, lo, hi);
    butterfly_rows<16>(lo);
    butterfly_rows<16>(hi);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const float* v = half ? hi : lo;
#pragma unroll
      for (int r = 0; r < 16; ++r) xch[(wave * 16 + r) * 64 + lane] = v[r];
      __syncthreads();
      const float m = cross_group_stages<kD / 16, false>(xch, wave, lane, tile_groups);
      if (col_ok) f_rot = fmaxf(f_rot, m);
      __syncthreads();
    }
  }
  // the normalisation is applied once to the maximum: max_i fl(c v_i) = fl(c max_i v_i)
  const uint32_t m_rot = wave_max_u32(__float_as_uint(rht_norm<kD>() * f_rot));
  if (lane == 0) {
    red[0][wave] = m_raw;
    red[1][wave] = m_rot;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t nwg = gridDim.x * gridDim.y, wg = blockIdx.y * gridDim.x + blockIdx.x;
    uint32_t a = 0, b = 0;
    for (int w = 0; w < 8; ++w) {
      a = max(a, red[0][w]);
      b = max(b, red[1][w]);
    }
    ws[kWsHeader + wg] = a;
    ws[kWsHeader + nwg + wg] = b;
  }
}

// ---------------------------------------------------------------- pass 2: cast
template <bool kRow, int kD, bool kSR>
__global__ __launch_bounds__(kWideThreads) void cast_wide_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ld, const uint32_t* __restrict__ ws,
    uint4 sign_words, uint32_t key0, uint32_t key1, uint8_t* __restrict__ row_codes, uint8_t* __restrict__ row_scales,
    float* __restrict__ row_ts, uint8_t* __restrict__ col_codes, uint8_t* __restrict__ col_scales,
    float* __restrict__ col_ts) {
  __shared__ __attribute__((aligned(16))) uint8_t st_col_codes[kColCodesBytes];
  __shared__ __attribute__((aligned(16))) uint8_t st_col_scales[kColScalesBytes];
  __shared__ __attribute__((aligned(16))) uint8_t st_row_scales[kRow ? kRowScalesBytes : 16];
  __shared__ float lut_row[128], lut_col[128];
  __shared__ float xch[8 * 16 * 64];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t colblk = static_cast<int64_t>(blockIdx.x) * kWaveCols;
  const int64_t col0 = colblk + lane * 8;
  const int64_t group0 = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock, group = group0 + wave;
  const int64_t ngroups = rows / 16;
  const int tile_groups = static_cast<int>(min<int64_t>(kGroupsPerBlock, ngroups - group0));
  const bool active = col0 < cols && group < ngroups;
  const int64_t row0 = group * 16;

  // App. B.1 Eq. 1, from the maxima of pass 1 (raw tensor for the row copy, rotated tensor for the col copy).
  const float amax_raw = __uint_as_float(ws[0]), amax_col = __uint_as_float(ws[1]);
  float s_enc_r, s_dec_r, s_enc_c, s_dec_c;
  tensor_scales(amax_raw, s_enc_r, s_dec_r);
  tensor_scales(amax_col, s_enc_c, s_dec_c);
  if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) {
    if (kRow) { row_ts[0] = s_dec_r; row_ts[1] = amax_raw; }
    col_ts[0] = s_dec_c;
    col_ts[1] = amax_col;
  }
  if (tid < 256) {   // "real" block encode scale 1 / (fp32(code) * s_dec) for each stored code (App. B.2)
    const int code = tid & 127;
    const float den = e4m3_decode(code) * (tid < 128 ? s_dec_r : s_dec_c);
    const float inv = (den == 0.0f || code == 127) ? 0.0f : 1.0f / den;
    if (tid < 128) lut_row[code] = inv; else lut_col[code] = inv;
  }
  __syncthreads();

  Patch p;
  if (active) {
    load_patch(x, ld, row0, col0, p);
  } else {
#pragma unroll
    for (int r = 0; r < 16; ++r) p.raw[r] = make_uint4(0u, 0u, 0u, 0u);
  }
  uint32_t rnd[16][4];
  if (kSR && active) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      philox4x32_10(static_cast<uint32_t>(col0 >> 3), static_cast<uint32_t>(row0 + r), 0u, 0u, key0, key1, rnd[r]);
  }
  if (kRow && active)
    row_pass<kSR, false>(p, rnd, lane, wave, s_enc_r, lut_row, 0.0f, 0u, row_codes + row0 * (cols / 2) + col0 / 2, cols / 2,
                         st_row_scales);

  const uint32_t signs = group_signs<kD>(sign_words, group);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    float lo[16], hi[16];
    signed_column_pair(p, t, signs, lo, hi);
    butterfly_rows<16>(lo);
    butterfly_rows<16>(hi);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      float (&v)[16] = half ? hi : lo;
#pragma unroll
      for (int r = 0; r < 16; ++r) xch[(wave * 16 + r) * 64 + lane] = v[r];
      __syncthreads();
      cross_group_stages<kD / 16, true>(xch, wave, lane, tile_groups);
      __syncthreads();
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = rht_norm<kD>() * xch[(wave * 16 + r) * 64 + lane];
      if (active)
        emit_column<kSR, false>(v, 2 * t + half, rnd, lane, wave, s_enc_c, lut_col, 0.0f, 0u, st_col_codes, st_col_scales);
    }
  }
  __syncthreads();
  write_back_tile<kRow, true, kWideThreads>(tid, rows, cols, group0, ngroups, colblk, st_col_codes, st_col_scales,
                                            st_row_scales, row_scales, col_codes, col_scales);
}

template <bool kRow, int kD>
void launch_wide(const QuantizeArgs& a, dim3 grid, hipStream_t s) {
  const uint16_t* x = static_cast<const uint16_t*>(a.x);
  const uint4 signs = make_uint4(a.sign_words[0], a.sign_words[1], a.sign_words[2], a.sign_words[3]);
  if (a.do_amax) {
    hipLaunchKernelGGL((amax_wide_kernel<kD>), grid, dim3(kWideThreads), 0, s, x, a.rows, a.cols, a.ld, signs, a.ws);
    hipLaunchKernelGGL(amax_finalize_kernel, dim3(1), dim3(1024), 0, s, a.ws, grid.x * grid.y, a.amax_copy);
  }
  if (!a.do_cast) return;
  if (a.sr)
    hipLaunchKernelGGL((cast_wide_kernel<kRow, kD, true>), grid, dim3(kWideThreads), 0, s, x, a.rows, a.cols, a.ld, a.ws, signs,
                       a.key0, a.key1, a.row_codes, a.row_scales, a.row_ts, a.col_codes, a.col_scales, a.col_ts);
  else
    hipLaunchKernelGGL((cast_wide_kernel<kRow, kD, false>), grid, dim3(kWideThreads), 0, s, x, a.rows, a.cols, a.ld, a.ws, signs,
                       a.key0, a.key1, a.row_codes, a.row_scales, a.row_ts, a.col_codes, a.col_scales, a.col_ts);
}

}  // namespace

hipError_t launch_quantize_wide(const QuantizeArgs& a, hipStream_t s) {
  if (!a.want_col || a.block2d || (a.rht_dim != 32 && a.rht_dim != 128) || a.rows % a.rht_dim) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>((a.cols + kWaveCols - 1) / kWaveCols),
                  static_cast<unsigned>((a.rows / 16 + kGroupsPerBlock - 1) / kGroupsPerBlock));
  if (a.rht_dim == 32) {
    if (a.want_row) launch_wide<true, 32>(a, grid, s);
    else launch_wide<false, 32>(a, grid, s);
  } else {
    if (a.want_row) launch_wide<true, 128>(a, grid, s);
    else launch_wide<false, 128>(a, grid, s);
  }
  return hipGetLastError();
}

}  // namespace nvfp4
