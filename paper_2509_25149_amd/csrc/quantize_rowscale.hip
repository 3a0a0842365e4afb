// NVFP4 quantizer for gfx950 with a tensor-level scale of finer granularity (App. B.1, last sentence: the global
// scale may span a row instead of the whole tensor, which saves the extra pass over device memory).
//
// The granularity is the one App. B.3 Eq. 5 lets the GEMM keep outside its sum over k: one FP32 scale per row of the
// copy's K-contiguous storage -- per logical row for the row copy, per logical column (in the rotated space, App. C)
// for the col copy.  Eq. 1 is evaluated per row with that row's amax; Eq. 2-4 are unchanged.
//
//   row copy alone    ONE pass over the tensor: a wavefront (rows of up to 8192 columns) or a workgroup (up to 32768)
//                     owns one row, holds all of it in registers, reduces the row's amax and encodes from the
//                     registers.  The bf16 tensor crosses HBM once.
//   col copy (+ row)  a column's amax spans every row of the tensor (all tokens), far more than a workgroup can hold,
//                     so this stays two passes, on the 16-row x 8-column lane patch of quantize.hip: pass 1 takes the
//                     maxima per row and per column (reduced inside the workgroup, then one atomic max per row /
//                     column and workgroup: 40 - 64 atomics per address at the 12B shapes), a small kernel turns them
//                     into the scale vectors, pass 2 encodes both copies.  The per-block "real" encode scale of
//                     App. B.2 is a division per block here: the 127-entry table of the per-tensor kernels would be
//                     a table per row.
#include "nvfp4_internal.h"
#include "quantize_tile.h"

namespace nvfp4 {

namespace {

// "real" block encode scale of App. B.2: 1 / (fp32(stored scale) * s_dec), 0 for a stored scale of 0
__device__ __forceinline__ float real_encode_scale(uint32_t code, float s_dec) {
  const float den = e4m3_decode(code) * s_dec;
  return den == 0.0f ? 0.0f : 1.0f / den;
}

typedef unsigned short ushort2p __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  union U {
    uint32_t u;
    ushort2p v;
  } x, y;
  x.u = a;
  y.u = b;
  x.v = __builtin_elementwise_max(x.v, y.v);
  return x.u;
}

// ---------------------------------------------------------------- row copy alone: one pass
// One workgroup per row; thread t holds the eight columns (ch * 256 + t) * 8 .. + 7 of every chunk ch < kNCH.
template <bool kSR, int kNCH>
__global__ __launch_bounds__(256) void rowscale_row_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                           int64_t ld, uint32_t key0, uint32_t key1,
                                                           uint8_t* __restrict__ row_codes, uint8_t* __restrict__ row_scales,
                                                           float* __restrict__ row_ts) {
  __shared__ uint32_t red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x;
  const uint16_t* xr = x + row * ld;

  uint4 raw[kNCH];
#pragma unroll
  for (int ch = 0; ch < kNCH; ++ch) {
    const int64_t col = (static_cast<int64_t>(ch) * 256 + tid) * 8;
    raw[ch] = col < cols ? *reinterpret_cast<const uint4*>(xr + col) : make_uint4(0u, 0u, 0u, 0u);
  }
  // the row's amax: bf16 magnitudes order like 15-bit integers, two per dword
  uint32_t m = 0u;
#pragma unroll
  for (int ch = 0; ch < kNCH; ++ch) {
    m = pk_max_u16(m, raw[ch].x & 0x7FFF7FFFu);
    m = pk_max_u16(m, raw[ch].y & 0x7FFF7FFFu);
    m = pk_max_u16(m, raw[ch].z & 0x7FFF7FFFu);
    m = pk_max_u16(m, raw[ch].w & 0x7FFF7FFFu);
  }
  m = wave_max_u32(max(m & 0xFFFFu, m >> 16));
  if (lane == 0) red[wave] = m;
  __syncthreads();
  const float amax = __uint_as_float(max(max(red[0], red[1]), max(red[2], red[3])) << 16);
  float s_enc, s_dec;
  tensor_scales(amax, s_enc, s_dec);                         // App. B.1 Eq. 1 with this row's amax
  if (tid == 0) {
    row_ts[row] = s_dec;
    row_ts[rows + row] = amax;
  }

  uint8_t* codes = row_codes + row * (cols / 2);
  uint8_t* scales = row_scales + row * (cols / 16);
#pragma unroll
  for (int ch = 0; ch < kNCH; ++ch) {
    const int64_t col = (static_cast<int64_t>(ch) * 256 + tid) * 8;
    if ((static_cast<int64_t>(ch) * 256 + (tid & ~63)) * 8 >= cols) break;   // the whole wavefront is past the end
    float v[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = patch_elem(raw[ch], c);
    float bm = 0.0f;
#pragma unroll
    for (int c = 0; c < 8; ++c) bm = fmaxf(bm, fabsf(v[c]));
    bm = fmaxf(bm, lane_xor1(bm));                           // the block is this lane's eight columns and the neighbour's
    const uint32_t code = e4m3_encode(div_by_6(bm) * s_enc);  // Eq. 2-3
    const float s_enc_b = real_encode_scale(code, s_dec);
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] *= s_enc_b;              // Eq. 4
    uint32_t rnd[4] = {0u, 0u, 0u, 0u};
    if (kSR) philox4x32_10(static_cast<uint32_t>(col >> 3), static_cast<uint32_t>(row), 0u, 0u, key0, key1, rnd);
    const uint32_t d = encode8<kSR>(v, rnd);
    if (col < cols) {
      *reinterpret_cast<uint32_t*>(codes + col / 2) = d;
      if ((lane & 1) == 0) scales[col / 16] = static_cast<uint8_t>(code);
    }
  }
}

// Rows of up to 8192 columns: one WAVEFRONT per row (four rows per workgroup), lane l holds the eight columns
// (ch * 64 + l) * 8 .. + 7 of every chunk ch < kNCH.  No LDS and no barrier, and several 16-byte loads in flight
// per lane: for short rows the workgroup-per-row form above spends its time on launches and its one barrier.
template <bool kSR, int kNCH>
__global__ __launch_bounds__(256) void rowscale_row_wave_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                                int64_t ld, uint32_t key0, uint32_t key1,
                                                                uint8_t* __restrict__ row_codes, uint8_t* __restrict__ row_scales,
                                                                float* __restrict__ row_ts) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (row >= rows) return;
  const uint16_t* xr = x + row * ld;
  uint4 raw[kNCH];
#pragma unroll
  for (int ch = 0; ch < kNCH; ++ch) {
    const int64_t col = (static_cast<int64_t>(ch) * 64 + lane) * 8;
    raw[ch] = col < cols ? *reinterpret_cast<const uint4*>(xr + col) : make_uint4(0u, 0u, 0u, 0u);
  }
  uint32_t m = 0u;
#pragma unroll
  for (int ch = 0; ch < kNCH; ++ch) {
    m = pk_max_u16(m, raw[ch].x & 0x7FFF7FFFu);
    m = pk_max_u16(m, raw[ch].y & 0x7FFF7FFFu);
    m = pk_max_u16(m, raw[ch].z & 0x7FFF7FFFu);
    m = pk_max_u16(m, raw[ch].w & 0x7FFF7FFFu);
  }
  const float amax = __uint_as_float(wave_max_u32(max(m & 0xFFFFu, m >> 16)) << 16);
  float s_enc, s_dec;
  tensor_scales(amax, s_enc, s_dec);                         // App. B.1 Eq. 1 with this row's amax
  if (lane == 0) {
    row_ts[row] = s_dec;
    row_ts[rows + row] = amax;
  }
  uint8_t* codes = row_codes + row * (cols / 2);
  uint8_t* scales = row_scales + row * (cols / 16);
#pragma unroll
  for (int ch = 0; ch < kNCH; ++ch) {
    const int64_t col = (static_cast<int64_t>(ch) * 64 + lane) * 8;
    if (static_cast<int64_t>(ch) * 512 >= cols) break;       // the whole wavefront is past the end
    float v[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = patch_elem(raw[ch], c);
    float bm = 0.0f;
#pragma unroll
    for (int c = 0; c < 8; ++c) bm = fmaxf(bm, fabsf(v[c]));
    bm = fmaxf(bm, lane_xor1(bm));
    const uint32_t code = e4m3_encode(div_by_6(bm) * s_enc);  // Eq. 2-3
    const float s_enc_b = real_encode_scale(code, s_dec);
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] *= s_enc_b;              // Eq. 4
    uint32_t rnd[4] = {0u, 0u, 0u, 0u};
    if (kSR) philox4x32_10(static_cast<uint32_t>(col >> 3), static_cast<uint32_t>(row), 0u, 0u, key0, key1, rnd);
    const uint32_t d = encode8<kSR>(v, rnd);
    if (col < cols) {
      *reinterpret_cast<uint32_t*>(codes + col / 2) = d;
      if ((lane & 1) == 0) scales[col / 16] = static_cast<uint8_t>(code);
    }
  }
}

// ---------------------------------------------------------------- both copies (or the col copy): two passes
// Workspace words: [0, rows) row amax bits, [rows, rows + cols) col amax bits, then the same two runs again holding
// the encode scales s_enc.
__global__ __launch_bounds__(256) void rowscale_zero_kernel(uint32_t* __restrict__ ws, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) ws[i] = 0u;
}

template <bool kRow, bool kCol, int kRht>
__global__ __launch_bounds__(kThreads) void rowscale_amax_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                                 int64_t ld, uint32_t sign_mask, uint32_t* __restrict__ ws) {
  __shared__ float col_max[kCol ? kGroupsPerBlock : 1][kWaveCols];   // [group in the tile][column of the tile]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t colblk = static_cast<int64_t>(blockIdx.x) * kWaveCols;
  const int64_t col0 = colblk + lane * 8;
#pragma unroll 1
  for (int gi = 0; gi < kGroupsPerWave; ++gi) {
    const int gl = wave * kGroupsPerWave + gi;
    const int64_t group = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock + gl;
    const bool live = group * 16 < rows;                    // wave-uniform
    Patch p;
    if (live && col0 < cols) {
      load_patch(x, ld, group * 16, col0, p);
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) p.raw[r] = make_uint4(0u, 0u, 0u, 0u);
    }
    if (kRow && live) {
      // rows 2d, 2d + 1 of the group share dword d: the lane's maxima as 16-bit magnitudes, then across the wavefront
      uint32_t rm[8];
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        uint32_t pair = 0u;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const uint4 q = p.raw[2 * d + h];
          uint32_t m = pk_max_u16(pk_max_u16(q.x & 0x7FFF7FFFu, q.y & 0x7FFF7FFFu), pk_max_u16(q.z & 0x7FFF7FFFu, q.w & 0x7FFF7FFFu));
          m = max(m & 0xFFFFu, m >> 16);
          pair |= m << (16 * h);
        }
        rm[d] = pair;
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1)
#pragma unroll
        for (int d = 0; d < 8; ++d) rm[d] = pk_max_u16(rm[d], static_cast<uint32_t>(__shfl_xor(static_cast<int>(rm[d]), off, 64)));
#pragma unroll
      for (int d = 0; d < 8; ++d)
        if (lane == d) {
          atomicMax(ws + group * 16 + 2 * d, (rm[d] & 0xFFFFu) << 16);
          atomicMax(ws + group * 16 + 2 * d + 1, rm[d] & 0xFFFF0000u);
        }
    }
    if (kCol) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float lo[16], hi[16];
        signed_column_pair(p, t, sign_mask, lo, hi);
        if (kRht) {
          butterfly_rows<kRht == 0 ? 1 : kRht>(lo);
          butterfly_rows<kRht == 0 ? 1 : kRht>(hi);
        }
        float ml = 0.0f, mh = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          ml = fmaxf(ml, fabsf(lo[r]));
          mh = fmaxf(mh, fabsf(hi[r]));
        }
        // the normalisation once, on the maximum: rounding is monotone, max_i fl(c v_i) = fl(c max_i v_i)
        if (kRht) {
          ml *= rht_norm<kRht == 0 ? 16 : kRht>();
          mh *= rht_norm<kRht == 0 ? 16 : kRht>();
        }
        col_max[gl][lane * 8 + 2 * t] = ml;
        col_max[gl][lane * 8 + 2 * t + 1] = mh;
      }
    }
  }
  if (kCol) {
    __syncthreads();
    for (int j = tid; j < kWaveCols; j += kThreads) {
      float m = 0.0f;
#pragma unroll
      for (int g = 0; g < kGroupsPerBlock; ++g) m = fmaxf(m, col_max[g][j]);
      if (colblk + j < cols) atomicMax(ws + rows + colblk + j, __float_as_uint(m));   // non-negative floats order like integers
    }
  }
}

// amax vectors -> Eq. 1 per row: encode scales into the workspace, decode scales and maxima into tensor_scale
__global__ __launch_bounds__(256) void rowscale_scales_kernel(uint32_t* __restrict__ ws, int64_t rows, int64_t cols,
                                                              float* __restrict__ row_ts, float* __restrict__ col_ts) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= rows + cols) return;
  const float amax = __uint_as_float(ws[i]);
  float s_enc, s_dec;
  tensor_scales(amax, s_enc, s_dec);
  ws[rows + cols + i] = __float_as_uint(s_enc);
  if (i < rows) {
    if (row_ts) {
      row_ts[i] = s_dec;
      row_ts[rows + i] = amax;
    }
  } else if (col_ts) {
    col_ts[i - rows] = s_dec;
    col_ts[cols + i - rows] = amax;
  }
}

template <bool kRow, bool kCol, int kRht, bool kSR>
__global__ __launch_bounds__(kThreads, 2) void rowscale_cast_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ld, const uint32_t* __restrict__ ws,
    uint32_t sign_mask, uint32_t key0, uint32_t key1, uint8_t* __restrict__ row_codes, uint8_t* __restrict__ row_scales,
    const float* __restrict__ row_ts, uint8_t* __restrict__ col_codes, uint8_t* __restrict__ col_scales,
    const float* __restrict__ col_ts) {
  __shared__ __attribute__((aligned(16))) uint8_t st_col_codes[kCol ? kColCodesBytes : 16];
  __shared__ __attribute__((aligned(16))) uint8_t st_col_scales[kCol ? kColScalesBytes : 16];
  __shared__ __attribute__((aligned(16))) uint8_t st_row_scales[kRow ? kRowScalesBytes : 16];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t colblk = static_cast<int64_t>(blockIdx.x) * kWaveCols;
  const int64_t col0 = colblk + lane * 8;
  const int64_t group0 = static_cast<int64_t>(blockIdx.y) * kGroupsPerBlock;
  const int64_t ngroups = rows / 16;
  const float* senc_row = reinterpret_cast<const float*>(ws) + rows + cols;
  const float* senc_col = senc_row + rows;

  // this lane's eight columns: encode and decode scale of each (Eq. 1 per column of the tensor)
  float s_enc_c[8], s_dec_c[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const bool in = kCol && col0 + c < cols;
    s_enc_c[c] = in ? senc_col[col0 + c] : 1.0f;
    s_dec_c[c] = in ? col_ts[col0 + c] : 1.0f;
  }

#pragma unroll 1
  for (int gi = 0; gi < kGroupsPerWave; ++gi) {
    const int gl = wave * kGroupsPerWave + gi;
    const int64_t group = group0 + gl;
    if (group >= ngroups) continue;                          // wave-uniform
    const int64_t row0 = group * 16;
    Patch p;
    if (col0 < cols) {
      load_patch(x, ld, row0, col0, p);
    } else {                                                 // lanes past the last column run along on zeros and store nothing
#pragma unroll
      for (int r = 0; r < 16; ++r) p.raw[r] = make_uint4(0u, 0u, 0u, 0u);
    }
    const bool in = col0 < cols;

    uint32_t rnd[16][4];
    if (kSR) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        philox4x32_10(static_cast<uint32_t>(col0 >> 3), static_cast<uint32_t>(row0 + r), 0u, 0u, key0, key1, rnd[r]);
    }

    if (kRow) {
      uint8_t* dst = row_codes + row0 * (cols / 2) + col0 / 2;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float s_enc_r = senc_row[row0 + r], s_dec_r = row_ts[row0 + r];   // the row's scales: the same for the whole wavefront
        float v[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] = patch_elem(p.raw[r], c);
        float m = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) m = fmaxf(m, fabsf(v[c]));
        m = fmaxf(m, lane_xor1(m));
        const uint32_t code = e4m3_encode(div_by_6(m) * s_enc_r);   // Eq. 2-3
        const float s_enc_b = real_encode_scale(code, s_dec_r);
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] *= s_enc_b;                // Eq. 4
        const uint32_t d = encode8<kSR>(v, rnd[r]);
        if (in) *reinterpret_cast<uint32_t*>(dst + r * (cols / 2)) = d;
        if ((lane & 1) == 0) st_row_scales[(gl * 16 + r) * 32 + (lane >> 1)] = static_cast<uint8_t>(code);
      }
    }

    if (kCol) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float lo[16], hi[16];
        signed_column_pair(p, t, sign_mask, lo, hi);
        if (kRht) {
          butterfly_rows<kRht == 0 ? 1 : kRht>(lo);
          butterfly_rows<kRht == 0 ? 1 : kRht>(hi);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            lo[r] *= rht_norm<kRht == 0 ? 16 : kRht>();
            hi[r] *= rht_norm<kRht == 0 ? 16 : kRht>();
          }
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          float(&v)[16] = h ? hi : lo;
          const int c = 2 * t + h;
          float m = 0.0f;
#pragma unroll
          for (int r = 0; r < 16; r += 2) m = fmaxf(fmaxf(m, fabsf(v[r])), fabsf(v[r + 1]));
          const uint32_t code = e4m3_encode(div_by_6(m) * s_enc_c[c]);
          const float s_enc_b = real_encode_scale(code, s_dec_c[c]);
#pragma unroll
          for (int r = 0; r < 16; ++r) v[r] *= s_enc_b;
          uint2 out;
          out.x = encode8_col<kSR>(v, rnd, 0, c);
          out.y = encode8_col<kSR>(v + 8, rnd, 8, c);
          *reinterpret_cast<uint2*>(st_col_codes + ((c * kGroupsPerBlock + gl) * kColSlot + lane) * 8) = out;
          st_col_scales[(c * kGroupsPerBlock + gl) * 64 + lane] = static_cast<uint8_t>(code);
        }
      }
    }
  }
  __syncthreads();
  write_back_tile<kRow, kCol, kThreads>(tid, rows, cols, group0, ngroups, colblk, st_col_codes, st_col_scales, st_row_scales,
                                          row_scales, col_codes, col_scales);
}

template <bool kSR, int kNCH>
void launch_row(const QuantizeArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((rowscale_row_kernel<kSR, kNCH>), dim3(static_cast<unsigned>(a.rows)), dim3(256), 0, s,
                     static_cast<const uint16_t*>(a.x), a.rows, a.cols, a.ld, a.key0, a.key1, a.row_codes, a.row_scales, a.row_ts);
}

template <bool kSR, int kNCH>
void launch_row_wave(const QuantizeArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((rowscale_row_wave_kernel<kSR, kNCH>), dim3(static_cast<unsigned>((a.rows + 3) / 4)), dim3(256), 0, s,
                     static_cast<const uint16_t*>(a.x), a.rows, a.cols, a.ld, a.key0, a.key1, a.row_codes, a.row_scales, a.row_ts);
}

template <bool kRow, bool kCol, int kRht>
void launch_two_pass(const QuantizeArgs& a, hipStream_t s) {
  const uint16_t* x = static_cast<const uint16_t*>(a.x);
  const dim3 grid(static_cast<unsigned>((a.cols + kWaveCols - 1) / kWaveCols),
                  static_cast<unsigned>((a.rows / 16 + kGroupsPerBlock - 1) / kGroupsPerBlock));
  const int64_t n = a.rows + a.cols;
  const unsigned nblk = static_cast<unsigned>((n + 255) / 256);
  hipLaunchKernelGGL(rowscale_zero_kernel, dim3(nblk), dim3(256), 0, s, a.ws, n);
  hipLaunchKernelGGL((rowscale_amax_kernel<kRow, kCol, kRht>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.sign_mask, a.ws);
  hipLaunchKernelGGL(rowscale_scales_kernel, dim3(nblk), dim3(256), 0, s, a.ws, a.rows, a.cols, kRow ? a.row_ts : nullptr,
                     kCol ? a.col_ts : nullptr);
  if (a.sr)
    hipLaunchKernelGGL((rowscale_cast_kernel<kRow, kCol, kRht, true>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.ws,
                       a.sign_mask, a.key0, a.key1, a.row_codes, a.row_scales, a.row_ts, a.col_codes, a.col_scales, a.col_ts);
  else
    hipLaunchKernelGGL((rowscale_cast_kernel<kRow, kCol, kRht, false>), grid, dim3(kThreads), 0, s, x, a.rows, a.cols, a.ld, a.ws,
                       a.sign_mask, a.key0, a.key1, a.row_codes, a.row_scales, a.row_ts, a.col_codes, a.col_scales, a.col_ts);
}

}  // namespace

// Words of workspace the two-pass form needs: amax and encode scale per row and per column.
size_t quantize_rowscale_workspace_words(int64_t rows, int64_t cols) { return static_cast<size_t>(2 * (rows + cols)); }

hipError_t launch_quantize_rowscale(const QuantizeArgs& a, hipStream_t s) {
  if (a.want_row && !a.want_col && a.cols <= 8192) {         // the row fits a wavefront's registers: one pass
    const int64_t nch = (a.cols + 511) / 512;
    if (a.sr) {
      if (nch <= 2) launch_row_wave<true, 2>(a, s);
      else if (nch <= 4) launch_row_wave<true, 4>(a, s);
      else if (nch <= 10) launch_row_wave<true, 10>(a, s);
      else launch_row_wave<true, 16>(a, s);
    } else {
      if (nch <= 2) launch_row_wave<false, 2>(a, s);
      else if (nch <= 4) launch_row_wave<false, 4>(a, s);
      else if (nch <= 10) launch_row_wave<false, 10>(a, s);
      else launch_row_wave<false, 16>(a, s);
    }
    return hipGetLastError();
  }
  if (a.want_row && !a.want_col && a.cols <= 32768) {        // the row fits a workgroup's registers: one pass
    const int64_t nch = (a.cols + 2047) / 2048;
    if (a.sr) {
      if (nch <= 2) launch_row<true, 2>(a, s);
      else if (nch <= 4) launch_row<true, 4>(a, s);
      else if (nch <= 10) launch_row<true, 10>(a, s);
      else launch_row<true, 16>(a, s);
    } else {
      if (nch <= 2) launch_row<false, 2>(a, s);
      else if (nch <= 4) launch_row<false, 4>(a, s);
      else if (nch <= 10) launch_row<false, 10>(a, s);
      else launch_row<false, 16>(a, s);
    }
    return hipGetLastError();
  }
  const bool rht = a.want_col && a.rht_dim == 16;
  if (a.want_row && a.want_col) {
    if (rht) launch_two_pass<true, true, 16>(a, s); else launch_two_pass<true, true, 0>(a, s);
  } else if (a.want_col) {
    if (rht) launch_two_pass<false, true, 16>(a, s); else launch_two_pass<false, true, 0>(a, s);
  } else {
    launch_two_pass<true, false, 0>(a, s);
  }
  return hipGetLastError();
}

}  // namespace nvfp4
