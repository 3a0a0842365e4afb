// Output stage shared by the 4-wavefront GEMM kernels for gfx950: one wavefront's 128 x 128 block of FP32 sums,
// held as 8 x 8 results of 16x16 MFMAs (acc[i][j][r] = D[m = 16 i + (lane & 15)][n = 16 j + 4 (lane >> 4) + r]),
// times the tensor-level decode scales (App. B.3, after Eq. 5), to FP32 (optionally added into D) or bf16.
// Device code only.
#pragma once

#include "nvfp4_device.h"

namespace nvfp4 {

// row0 / col0: the block's first row / column in D; rows / cols: how many of its 128 x 128 exist (multiples of 16,
// possibly <= 0).  Stored from the registers: a lane writes its 4 consecutive columns of one row, 16 bytes (FP32) or
// 8 bytes (bf16).  (Reordering the bf16 block through LDS into 256-byte row pieces was tried and measured no
// faster: what the stage costs is the burst of all workgroups finishing their tiles together, not its shape.)
template <bool kBf16Out>
__device__ __forceinline__ void store_wave_block(float4v (&acc)[8][8], float out_scale, void* __restrict__ Dv, int64_t ldd,
                                                 bool accumulate, int64_t row0, int64_t col0, int rows, int cols, int lane) {
  const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int m = i * 16 + l16;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int n = j * 16 + lq * 4;
      if (m < rows && n < cols) {  // columns come in multiples of 16, so the 4 columns are in or out together
        float4v v = acc[i][j] * out_scale;
        if (kBf16Out) {
          uint16_t* d = static_cast<uint16_t*>(Dv) + (row0 + m) * ldd + col0 + n;
          uint2 o;
          o.x = f32_to_bf16(v[0]) | (f32_to_bf16(v[1]) << 16);
          o.y = f32_to_bf16(v[2]) | (f32_to_bf16(v[3]) << 16);
          *reinterpret_cast<uint2*>(d) = o;
        } else {
          float* d = static_cast<float*>(Dv) + (row0 + m) * ldd + col0 + n;
          if (accumulate) v += *reinterpret_cast<const float4v*>(d);
          *reinterpret_cast<float4v*>(d) = v;
        }
      }
    }
  }
}

}  // namespace nvfp4
