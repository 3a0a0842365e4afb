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
#include "quantize_tile.h"

namespace nvfp4 {


// ---------------------------------------------------------------- pass 1: amax (App. B.1)
// Every workgroup writes its own maxima (raw tensor / rotated tensor) into its
// slot of the workspace; a one-workgroup kernel folds the slots.  No atomics:
// thousands of same-address atomics serialise in L2 and cost more than the pass.
// The raw maximum is always taken, also when only a rotated copy is asked for: it is the one place where a NaN in
// the input shows (the floating-point maxima of the rotated values skip NaNs), and amax_finalize_kernel carries a
// non-finite raw maximum over into the rotated one.
template <int kRht>   // kRht: 0, or the rotation size 2, 4 or 16 (sign_mask: the d signs repeated over 16 bits)
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
      m_raw = max(m_raw, patch_amax_bits(p));
      if (kRht) {
        // The normalisation is applied once to the maximum: rounding is monotone, so
        // max_i fl(c v_i) = fl(c max_i v_i).
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          float lo[16], hi[16];
          signed_column_pair(p, t, sign_mask, lo, hi);
          butterfly_rows<kRht>(lo);
          butterfly_rows<kRht>(hi);
#pragma unroll
          for (int r = 0; r < 16; ++r) f_rot = fmaxf(fmaxf(f_rot, fabsf(lo[r])), fabsf(hi[r]));
        }
      }
    }
  }
  m_raw = wave_max_u32(m_raw);
  if (kRht) m_rot = wave_max_u32(__float_as_uint(rht_norm<kRht>() * f_rot));
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

// ---------------------------------------------------------------- pass 2: cast



template <bool kRow, bool kCol, int kRht, bool kSR, bool k2D>   // kRht as in amax_kernel
__global__ __launch_bounds__(kThreads, 2) void cast_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ld,
    const uint32_t* __restrict__ ws, uint32_t sign_mask, uint32_t key0, uint32_t key1,
    uint8_t* __restrict__ row_codes, uint8_t* __restrict__ row_scales, float* __restrict__ row_ts,
    uint8_t* __restrict__ col_codes, uint8_t* __restrict__ col_scales, float* __restrict__ col_ts, int reverse) {
  __shared__ __attribute__((aligned(16))) uint8_t st_col_codes[kCol ? kColCodesBytes : 16];
  __shared__ __attribute__((aligned(16))) uint8_t st_col_scales[kCol ? kColScalesBytes : 16];
  __shared__ __attribute__((aligned(16))) uint8_t st_row_scales[kRow ? kRowScalesBytes : 16];
  __shared__ float lut_row[128], lut_col[128];  // block encode scale per stored E4M3 code

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const unsigned bx = reverse ? gridDim.x - 1 - blockIdx.x : blockIdx.x, by = reverse ? gridDim.y - 1 - blockIdx.y : blockIdx.y;
  const int64_t colblk = static_cast<int64_t>(bx) * kWaveCols;
  const int64_t col0 = colblk + lane * 8;
  const int64_t group0 = static_cast<int64_t>(by) * kGroupsPerBlock;
  const int64_t ngroups = rows / 16;

  // App. B.1 Eq. 1, from the amax of pass 1.
  const float amax_raw = __uint_as_float(ws[0]);
  const float amax_col = kRht ? __uint_as_float(ws[1]) : amax_raw;
  float s_enc_r, s_dec_r, s_enc_c, s_dec_c;
  tensor_scales(amax_raw, s_enc_r, s_dec_r);
  tensor_scales(amax_col, s_enc_c, s_dec_c);
  if (bx == 0 && by == 0 && tid == 0) {
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

    // (Requesting both patches of the wavefront up front was tried for the kernels without stochastic rounding, which
    // have the registers: 157 - 173 instead of 113 - 120 cost a wavefront per SIMD, and X / W went from 59 / 122 us per
    // call to 62 / 130.)
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
      m = max(m, lane_xor1(m));
      tile_code = e4m3_encode(div_by_6(__uint_as_float(m)) * s_enc_r);   // Eq. 2-3
      s_enc_tile = lut_row[tile_code];
    }

    if (kRow)
      row_pass<kSR, k2D>(p, rnd, lane, gl, s_enc_r, lut_row, s_enc_tile, tile_code, row_codes + row0 * (cols / 2) + col0 / 2,
                         cols / 2, st_row_scales);

    if (kCol) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float lo[16], hi[16];
        // Without a rotation sign_mask is 0 at run time; it is still applied, so that these values are not
        // recognised as the row pass's: keeping all 128 of those alive costs more registers than there are.
        signed_column_pair(p, t, sign_mask, lo, hi);
        if (kRht) {
          butterfly_rows<kRht>(lo);
          butterfly_rows<kRht>(hi);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            lo[r] *= rht_norm<kRht>();
            hi[r] *= rht_norm<kRht>();
          }
        }
        emit_column<kSR, k2D>(lo, 2 * t, rnd, lane, gl, s_enc_c, lut_col, s_enc_tile, tile_code, st_col_codes, st_col_scales);
        emit_column<kSR, k2D>(hi, 2 * t + 1, rnd, lane, gl, s_enc_c, lut_col, s_enc_tile, tile_code, st_col_codes, st_col_scales);
      }
    }
  }
  __syncthreads();

  write_back_tile<kRow, kCol, kThreads>(tid, rows, cols, group0, ngroups, colblk, st_col_codes, st_col_scales,
                                          st_row_scales, row_scales, col_codes, col_scales);
}

// ---------------------------------------------------------------- host side

size_t quantize_workspace_bytes(int64_t rows, int64_t cols) {
  const int64_t gx = (cols + kWaveCols - 1) / kWaveCols, gy = (rows / 16 + kGroupsPerBlock - 1) / kGroupsPerBlock;
  // raw, col-rotated, row-rotated maxima per workgroup; or, with one scale per row of each copy, amax and encode scale
  // per row and per column
  const size_t per_tensor = static_cast<size_t>(kWsHeader + 3 * gx * gy), per_row = quantize_rowscale_workspace_words(rows, cols);
  return (per_tensor > per_row ? per_tensor : per_row) * sizeof(uint32_t);
}

// The cast pass walks a large tensor from its end: the amax pass has just streamed it front to back, so its tail is
// what the 256 MB memory-side cache still holds (measured at the 12B shapes: W 124 -> 121 us, dY 250 -> 245 us per
// call; a tensor that fits the cache whole gains nothing either way).
static int cast_reverse(const QuantizeArgs& a) { return a.do_amax && a.rows * a.cols * 2 > (int64_t{128} << 20); }

template <bool kRow, bool kCol, int kRht, bool kSR, bool k2D>
static void launch_cast(const QuantizeArgs& a, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL((cast_kernel<kRow, kCol, kRht, kSR, k2D>), grid, dim3(kThreads), 0, s,
                     static_cast<const uint16_t*>(a.x), a.rows, a.cols, a.ld, a.ws, a.sign_mask, a.key0,
                     a.key1, a.row_codes, a.row_scales, a.row_ts, a.col_codes, a.col_scales, a.col_ts, cast_reverse(a));
}

template <bool kRow, bool kCol, int kRht>
static void dispatch_cast2(const QuantizeArgs& a, dim3 grid, hipStream_t s) {
  if (a.block2d) {
    if (a.sr) launch_cast<kRow, kCol, 0, true, true>(a, grid, s);
    else launch_cast<kRow, kCol, 0, false, true>(a, grid, s);
  } else {
    if (a.sr) launch_cast<kRow, kCol, kRht, true, false>(a, grid, s);
    else launch_cast<kRow, kCol, kRht, false, false>(a, grid, s);
  }
}

template <bool kRow, int kRht>
static void launch_rotated(const QuantizeArgs& a, dim3 grid, hipStream_t s) {
  const uint16_t* x = static_cast<const uint16_t*>(a.x);
  if (a.do_amax) {
    hipLaunchKernelGGL((amax_kernel<kRht>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.sign_mask, a.ws);
    hipLaunchKernelGGL(amax_finalize_kernel, dim3(1), dim3(1024), 0, s, a.ws, grid.x * grid.y, a.amax_copy);
  }
  if (a.do_cast) dispatch_cast2<kRow, true, kRht>(a, grid, s);
}

hipError_t launch_quantize(const QuantizeArgs& a, hipStream_t s) {
  const dim3 grid(static_cast<unsigned>((a.cols + kWaveCols - 1) / kWaveCols),
                  static_cast<unsigned>((a.rows / 16 + kGroupsPerBlock - 1) / kGroupsPerBlock));
  const int rht = a.want_col ? a.rht_dim : 0;
  if (a.scale_per_row) return launch_quantize_rowscale(a, s);
  if (a.row_rht) return launch_quantize_rowrot(a, s);
  if (rht > 16) return launch_quantize_wide(a, s);
  if (rht) {
    if (a.want_row) {
      if (rht == 16) launch_rotated<true, 16>(a, grid, s);
      else if (rht == 4) launch_rotated<true, 4>(a, grid, s);
      else launch_rotated<true, 2>(a, grid, s);
    } else {
      if (rht == 16) launch_rotated<false, 16>(a, grid, s);
      else if (rht == 4) launch_rotated<false, 4>(a, grid, s);
      else launch_rotated<false, 2>(a, grid, s);
    }
    return hipGetLastError();
  }
  if (a.do_amax) {
    hipLaunchKernelGGL((amax_kernel<0>), grid, dim3(kThreads), 0, s, static_cast<const uint16_t*>(a.x), a.rows, a.cols,
                       a.ld, a.sign_mask, a.ws);
    hipLaunchKernelGGL(amax_finalize_kernel, dim3(1), dim3(1024), 0, s, a.ws, grid.x * grid.y, a.amax_copy);
  }
  if (a.do_cast) {
    if (a.want_row && a.want_col) dispatch_cast2<true, true, 0>(a, grid, s);
    else if (a.want_row) dispatch_cast2<true, false, 0>(a, grid, s);
    else dispatch_cast2<false, true, 0>(a, grid, s);
  }
  return hipGetLastError();
}

}  // namespace nvfp4
