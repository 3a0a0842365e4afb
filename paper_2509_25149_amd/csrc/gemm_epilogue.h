// Output stage shared by the 4-wavefront GEMM kernels for gfx950: one wavefront's 128 x 128 block of FP32 sums,
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
// FP32 results (weight gradients: large, read again only by the optimizer) leave with non-temporal stores: lines
// left dirty in the caches are written back during whatever runs next, a bandwidth-bound kernel (the quantizer
// call after a Wgrad took 63 us behind ordinary stores, 60 us behind these, and the Wgrad itself 0.5 % less).
// bf16 results (activations and their gradients, which the caller reads next) use ordinary stores: non-temporal
// ones made the amax pass behind Fprop a third faster (96 -> 62 us) but Fprop itself 4 % slower -- every workgroup
// of a round finishes its tile at the same moment and the burst drains at memory speed instead of into the caches
// (12 % slower with 32-byte pieces).  Must be called by all 64 lanes.  (Reordering the bf16 block through LDS into
// 256-byte row pieces was tried with ordinary stores and measured no faster.)
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));

template <bool kBf16Out>
__device__ __forceinline__ void store_wave_block(float4v (&acc)[8][8], float out_scale, void* __restrict__ Dv, int64_t ldd,
                                                 bool accumulate, int64_t row0, int64_t col0, int rows, int cols, int lane) {
  const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int m = i * 16 + l16;
    if (kBf16Out) {
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        const float4v va = acc[i][j] * out_scale, vb = acc[i][j + 1] * out_scale;
        const uint32_t a0 = f32_to_bf16(va[0]) | (f32_to_bf16(va[1]) << 16), a1 = f32_to_bf16(va[2]) | (f32_to_bf16(va[3]) << 16);
        const uint32_t b0 = f32_to_bf16(vb[0]) | (f32_to_bf16(vb[1]) << 16), b1 = f32_to_bf16(vb[2]) | (f32_to_bf16(vb[3]) << 16);
        // first result: lanes of odd groups now hold the second block's dword of the group below; second result: lanes of
        // even groups now hold the first block's dword of the group above
        const auto s0 = __builtin_amdgcn_permlane16_swap(a0, b0, false, false);
        const auto s1 = __builtin_amdgcn_permlane16_swap(a1, b1, false, false);
        const u32x4v o = {s0[0], s1[0], s0[1], s1[1]};
        const int n = (lq & 1) ? (j + 1) * 16 + (lq - 1) * 4 : j * 16 + lq * 4;   // 8 columns from here
        if (m < rows && n < cols) {   // columns come in multiples of 16, so the 8 columns are in or out together
          uint16_t* d = static_cast<uint16_t*>(Dv) + (row0 + m) * ldd + col0 + n;
          *reinterpret_cast<u32x4v*>(d) = o;
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int n = j * 16 + lq * 4;
        if (m < rows && n < cols) {  // columns come in multiples of 16, so the 4 columns are in or out together
          float4v v = acc[i][j] * out_scale;
          float* d = static_cast<float*>(Dv) + (row0 + m) * ldd + col0 + n;
          if (accumulate) v += *reinterpret_cast<const float4v*>(d);
          __builtin_nontemporal_store(v, reinterpret_cast<float4v*>(d));
        }
      }
    }
  }
}

}  // namespace nvfp4
