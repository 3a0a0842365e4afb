// NVFP4 quantizer kernels for gfx950 (App. B Eq. 1-4; Sec. 4.2-4.4; App. C).
//
// Work decomposition shared by both passes: a lane owns a 16-row x 8-column
// patch of the bf16 tensor (sixteen 128-bit loads, one per row); a wavefront
// owns 16 rows x 512 columns, so each of its loads reads 1 KiB of contiguous
// memory; a 256-thread workgroup stacks four wavefronts on four consecutive
// 16-row groups.  With this patch
//   - a 1x16 block of the row copy is split over two neighbouring lanes
//     (one cross-lane exchange of the half-block amax),
//   - a 1x16 block of the col copy (16 consecutive rows of one column) sits
//     entirely in one lane's registers, so the Hadamard butterfly and the
//     block amax need no cross-lane traffic,
//   - a 16x16 weight tile is exactly two neighbouring lanes,
//   - the eight columns of one row are the eight elements served by one
//     Philox call, whose output is shared by the row and the col copy.
#include "nvfp4_internal.h"
#include "nvfp4_device.h"

namespace nvfp4 {

constexpr int kThreads = 256;
constexpr int kWaveCols = 512;     // 64 lanes x 8 columns
constexpr int kGroupsPerBlock = 4; // wavefronts per workgroup, one 16-row group each

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

// ---------------------------------------------------------------- pass 1: amax
// ws[0] = bits of max|x| ; ws[1] = bits of max|x rotated| (only if kRht).
template <bool kRaw, bool kRht>
__global__ __launch_bounds__(kThreads) void amax_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                        int64_t cols, int64_t ld, uint32_t sign_mask,
                                                        uint32_t* __restrict__ ws) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t col0 = static_cast<int64_t>(blockIdx.x) * kWaveCols + lane * 8;
  const int64_t group = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock + wave;
  uint32_t m_raw = 0, m_rot = 0;
  if (col0 < cols && group * 16 < rows) {
    Patch p;
    load_patch(x, ld, group * 16, col0, p);
    if (kRaw) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t w[4] = {p.raw[r].x, p.raw[r].y, p.raw[r].z, p.raw[r].w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          m_raw = max(m_raw, (w[t] << 16) & 0x7FFFFFFFu);
          m_raw = max(m_raw, w[t] & 0x7FFF0000u);
        }
      }
    }
    if (kRht) {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float v[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = patch_elem(p.raw[r], c);
        rht16(v, sign_mask);
#pragma unroll
        for (int r = 0; r < 16; ++r) m_rot = max(m_rot, __float_as_uint(v[r]) & 0x7FFFFFFFu);
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    if (kRaw) m_raw = max(m_raw, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m_raw), off, 64)));
    if (kRht) m_rot = max(m_rot, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m_rot), off, 64)));
  }
  if (lane == 0) {
    if (kRaw && m_raw) atomicMax(ws + 0, m_raw);
    if (kRht && m_rot) atomicMax(ws + 1, m_rot);
  }
}

__global__ void clear_ws_kernel(uint32_t* ws) {
  if (threadIdx.x < 4) ws[threadIdx.x] = 0u;
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

template <bool kRow, bool kCol, bool kRht, bool kSR, bool k2D>
__global__ __launch_bounds__(kThreads) void cast_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ld,
    const uint32_t* __restrict__ ws, uint32_t sign_mask, uint32_t key0, uint32_t key1,
    uint8_t* __restrict__ row_codes, uint8_t* __restrict__ row_scales, float* __restrict__ row_ts,
    uint8_t* __restrict__ col_codes, uint8_t* __restrict__ col_scales, float* __restrict__ col_ts) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t col0 = static_cast<int64_t>(blockIdx.x) * kWaveCols + lane * 8;
  const int64_t group = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock + wave;

  // App. B.1 Eq. 1, from the amax of pass 1.
  const float amax_raw = __uint_as_float(ws[0]);
  const float amax_col = kRht ? __uint_as_float(ws[1]) : amax_raw;
  float s_enc_r, s_dec_r, s_enc_c, s_dec_c;
  tensor_scales(amax_raw, s_enc_r, s_dec_r);
  tensor_scales(amax_col, s_enc_c, s_dec_c);
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
    if (kRow) { row_ts[0] = s_dec_r; row_ts[1] = amax_raw; }
    if (kCol) { col_ts[0] = s_dec_c; col_ts[1] = amax_col; }
  }
  if (col0 >= cols || group * 16 >= rows) return;
  const int64_t row0 = group * 16;

  Patch p;
  load_patch(x, ld, row0, col0, p);

  // Random words: one Philox call per row serves the row's 8 columns.
  uint32_t rnd[16][4];
  if (kSR) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      philox4x32_10(static_cast<uint32_t>(col0 >> 3), static_cast<uint32_t>(row0 + r), 0u, 0u, key0, key1,
                    rnd[r]);
  }

  // 16x16 tile amax (Sec. 4.3): this lane's 16x8 half and the neighbour's.
  float s_enc_tile = 0.0f;
  uint32_t tile_code = 0;
  if (k2D) {
    uint32_t m = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const uint32_t w[4] = {p.raw[r].x, p.raw[r].y, p.raw[r].z, p.raw[r].w};
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        m = max(m, (w[t] << 16) & 0x7FFFFFFFu);
        m = max(m, w[t] & 0x7FFF0000u);
      }
    }
    m = max(m, static_cast<uint32_t>(__shfl_xor(static_cast<int>(m), 1, 64)));
    s_enc_tile = block_scale(__uint_as_float(m), s_enc_r, s_dec_r, tile_code);
  }

  if (kRow) {
    const int64_t code_ld = cols / 2, scale_ld = cols / 16;
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
        s_enc_b = block_scale(m, s_enc_r, s_dec_r, code);
      }
#pragma unroll
      for (int c = 0; c < 8; ++c) v[c] *= s_enc_b;                  // Eq. 4
      const uint32_t d = encode8<kSR>(v, rnd[r]);
      *reinterpret_cast<uint32_t*>(row_codes + (row0 + r) * code_ld + col0 / 2) = d;
      if ((lane & 1) == 0) row_scales[(row0 + r) * scale_ld + col0 / 16] = static_cast<uint8_t>(code);
    }
  }

  if (kCol) {
    const int64_t code_ld = rows / 2, scale_ld = rows / 16;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      float v[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = patch_elem(p.raw[r], c);
      if (kRht) rht16(v, sign_mask);
      float s_enc_b;
      uint32_t code;
      if (k2D) {
        s_enc_b = s_enc_tile;
        code = tile_code;
      } else {
        float m = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) m = fmaxf(m, fabsf(v[r]));
        s_enc_b = block_scale(m, s_enc_c, s_dec_c, code);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] *= s_enc_b;
      uint32_t d0, d1;
      if (!kSR) {
        const uint32_t none[4] = {0, 0, 0, 0};
        d0 = encode8<false>(v, none);
        d1 = encode8<false>(v + 8, none);
      } else {
        const uint32_t e0 = merge_bytes(cvt_sr_single<0>(v[0], draw_hi16(rnd, 0, c)), cvt_sr_single<1>(v[2], draw_hi16(rnd, 2, c)),
                                        cvt_sr_single<2>(v[4], draw_hi16(rnd, 4, c)), cvt_sr_single<3>(v[6], draw_hi16(rnd, 6, c)));
        const uint32_t o0 = merge_bytes(cvt_sr_single<0>(v[1], draw_hi16(rnd, 1, c)), cvt_sr_single<1>(v[3], draw_hi16(rnd, 3, c)),
                                        cvt_sr_single<2>(v[5], draw_hi16(rnd, 5, c)), cvt_sr_single<3>(v[7], draw_hi16(rnd, 7, c)));
        const uint32_t e1 = merge_bytes(cvt_sr_single<0>(v[8], draw_hi16(rnd, 8, c)), cvt_sr_single<1>(v[10], draw_hi16(rnd, 10, c)),
                                        cvt_sr_single<2>(v[12], draw_hi16(rnd, 12, c)), cvt_sr_single<3>(v[14], draw_hi16(rnd, 14, c)));
        const uint32_t o1 = merge_bytes(cvt_sr_single<0>(v[9], draw_hi16(rnd, 9, c)), cvt_sr_single<1>(v[11], draw_hi16(rnd, 11, c)),
                                        cvt_sr_single<2>(v[13], draw_hi16(rnd, 13, c)), cvt_sr_single<3>(v[15], draw_hi16(rnd, 15, c)));
        d0 = interleave_nibbles(e0, o0);
        d1 = interleave_nibbles(e1, o1);
      }
      uint2 out;
      out.x = d0;
      out.y = d1;
      *reinterpret_cast<uint2*>(col_codes + (col0 + c) * code_ld + group * 8) = out;
      col_scales[(col0 + c) * scale_ld + group] = static_cast<uint8_t>(code);
    }
  }
}

// ---------------------------------------------------------------- host side

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
  hipLaunchKernelGGL(clear_ws_kernel, dim3(1), dim3(64), 0, s, a.ws);
  const bool rht = a.want_col && a.rht;
  const bool raw = a.want_row || !rht;
  const uint16_t* x = static_cast<const uint16_t*>(a.x);
  if (raw && rht)
    hipLaunchKernelGGL((amax_kernel<true, true>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.sign_mask, a.ws);
  else if (rht)
    hipLaunchKernelGGL((amax_kernel<false, true>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.sign_mask, a.ws);
  else
    hipLaunchKernelGGL((amax_kernel<true, false>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.sign_mask, a.ws);
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
