// NVFP4 CPU oracle -- TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, obviously-correct host implementation of the NVFP4
// quantize / dequantize / block-scaled GEMM path of "Pretraining Large
// Language Models with NVFP4" (arXiv 2509.25149).  It exists so the GPU
// library can be checked against something that was written from the paper
// and shares no code with it.  Nothing in the product path may call it: only
// the tests, the smoke check and the benchmark's cpu_baseline leg do.
//
// Build:  g++ -std=c++17 -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
// All floating point below is IEEE-754 binary32 with round-to-nearest-even,
// subnormals kept, no fused multiply-add (hence -ffp-contract=off), except the
// GEMM reference, which is binary64.  OpenMP only splits independent outer
// rows across cores; no arithmetic is reordered by it.
//
// What each routine follows:
//   formats            Sec. 2 (E2M1 value set; E4M3 block scale per 16
//                      elements; FP32 tensor scale), App. B.1 (maxima 6, 448)
//   quantization       App. B.1 Eq. 1, App. B.2 Eq. 2-3, App. B.3 Eq. 4
//   2D weight blocks   Sec. 4.3 "Block scaling"
//   Hadamard rotation  Sec. 4.2, App. C
//   stochastic round   Sec. 4.4
//   GEMM               Sec. 2 "Hardware support via Tensor Cores", App. B.3 Eq. 5
//
// Conventions the paper leaves open are fixed here (and mirrored by the GPU
// library, which implements them separately):
//   * E2M1 code = sign<<3 | index into {0, .5, 1, 1.5, 2, 3, 4, 6}.
//   * E4M3 is the 448-max variant: bias 7, subnormal step 2^-9, no infinity.
//   * Two codes per byte, even element in the low nibble.
//   * A "row" copy has its 16-element blocks along the columns of the
//     logical [rows, cols] tensor; a "col" copy is the row-wise quantization
//     of the transposed tensor (blocks along the logical rows) and is stored
//     transposed, [cols, rows/2] bytes.
//   * Ties in round-to-nearest go to the code whose mantissa bit is 0.
//   * |v| >= 6 saturates to 6.  The code's sign bit is the sign bit of the
//     scaled value, also when the magnitude rounds to zero.
//   * Stochastic rounding uses 16 random bits per element: with p the
//     position of |v| between its two grid neighbours (0 <= p < 1) the value
//     moves up iff floor(p * 2^16) + r >= 2^16.
//   * Random bits are Philox4x32-10 (Salmon et al., SC'11) keyed by the
//     64-bit seed; element (i, j) of the logical tensor uses counter
//     (j / 8, i, 0, 0), output word (j % 8) / 2, low half for even j.  Both
//     copies of a tensor therefore see the same draw for the same element.
//   * The Hadamard sign diagonal is the low 16 bits of word 0 of
//     Philox4x32-10(counter = (0, 0, 0, 0xFFFFFFFF), key = seed); bit i set
//     means s_i = -1.
//   * The 16-point transform is evaluated as y = H16 (s .* v) with the
//     butterfly stages h = 1, 2, 4, 8 in this order, then one multiply by
//     0.25; every add and subtract is one binary32 rounding.  The rotated
//     values stay in binary32 (no trip back to bf16) and the tensor amax of a
//     rotated copy is taken over the rotated values (App. C).
//   * Rotations of the other sizes the paper ablates (Sec. 4.2 "Hadamard
//     matrix size", App. E.4: d = 2, 4, 128; 32 for MXFP4) follow the same
//     construction: sign i is bit i of all 128 bits of that Philox call,
//     stages h = 1 .. d/2, then one multiply by the binary32 nearest to
//     1/sqrt(d); pinned (tests/test_oracle_rht_sizes.py) by the dense
//     Sylvester matrix, its closed-form entries, the even spread of a
//     single outlier, the amax the quantizer reports for such a tensor and
//     the invariance of the product; the bit-to-sign assignment is this
//     repository's convention (parity unpinned against the paper).
//   * A rotation always runs along the block direction of the copy being
//     quantized.  For a col copy that is the tensor's rows (the Wgrad
//     operands of the recipe); asked for on a row copy it is the tensor's
//     columns, the transform on the Fprop / Dgrad operands that App. E.4.1
//     ablates.  Pinned (tests/test_oracle_row_rotation.py) by the spread of
//     a single outlier along its row with the signs of the dense form, the
//     dense form of the stored values, the transposition identity with the
//     col copy, and the cancellation in Fprop and Dgrad.
//
//   * Tensor-level scale of finer granularity (App. B.1, last sentence: the
//     global scale may span a row or a block of elements instead of the whole
//     tensor, which saves the extra pass over memory).  The granularity taken
//     here is the one Eq. 5 allows the GEMM to pull out of the sum over k: one
//     FP32 scale per row of the copy's K-contiguous storage (per logical row
//     for a row copy, per logical column for a col copy).  Eq. 1 is evaluated
//     with that row's amax; Eq. 2-4 are unchanged.  Not combined with 16x16
//     blocks: a weight tile's scale must serve both orientations (Sec. 4.3).
//     Pinned (tests/test_oracle_row_scales.py) by a hand-worked two-row
//     tensor, by the row-by-row identity with the per-tensor routine, by the
//     0x7E scale of each row's amax block, by invariance of the codes under a
//     power-of-two scaling of single rows, and by the GEMM's closed forms.
//
// PARITY PINS (tests/test_oracle_*.py): E2M1/E4M3 by brute force over the whole
// code space; Philox by the published known-answer vectors; the transform by
// the dense matrix form, orthogonality and the GEMM-invariance identity of
// App. C; quantization by two hand-worked tensors (tests/golden), by the
// invariants of App. B.2 / Fig. 1, and by W / W^T identity for 2D blocks;
// SR by exhaustive sweeps of r and a many-seed mean; the GEMM by closed
// forms, integer cases and the Eq. 5 form.  The counter layout, sign-mask
// derivation, nibble order and sign-of-zero rule are conventions of this
// repository: parity unpinned against the paper (it states none), pinned
// oracle <-> GPU only.
// The MXFP4 section at the end of this file (the paper's comparison format) has
// its own header and pins (tests/test_oracle_mxfp4.py): the power-of-two
// round-up rule by exact rationals, the worked example of App. B.4, an
// independent numpy formulation, the no-saturation / lost-binade invariants,
// the 32-point Sylvester form, SR draws and unbiasedness.  Its draw counters
// for the col copy and its 32-bit sign vector are conventions of this
// repository (parity unpinned against the paper).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#include <limits>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// ---------------------------------------------------------------- formats

const float kE2M1Grid[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

inline float bf16_bits_to_f32(uint16_t h) {
  uint32_t w = static_cast<uint32_t>(h) << 16;
  float f;
  std::memcpy(&f, &w, 4);
  return f;
}

inline uint32_t f32_bits(float f) {
  uint32_t w;
  std::memcpy(&w, &f, 4);
  return w;
}

inline bool sign_bit(float f) { return (f32_bits(f) >> 31) != 0; }

float e2m1_decode(uint32_t code) {
  float m = kE2M1Grid[code & 7u];
  return (code & 8u) ? -m : m;
}

// Round-to-nearest onto the E2M1 grid; the midpoints between neighbours go
// to the neighbour with an even code (mantissa bit 0).  Sec. 4 item 4.
uint32_t e2m1_encode_rne(float v) {
  const float a = std::fabs(v);
  uint32_t idx;
  if (a <= 0.25f)      idx = 0;   // tie 0.25 -> 0
  else if (a < 0.75f)  idx = 1;
  else if (a <= 1.25f) idx = 2;   // ties 0.75 and 1.25 -> 1.0
  else if (a < 1.75f)  idx = 3;
  else if (a <= 2.5f)  idx = 4;   // ties 1.75 and 2.5 -> 2.0
  else if (a < 3.5f)   idx = 5;
  else if (a <= 5.0f)  idx = 6;   // ties 3.5 and 5.0 -> 4.0
  else                 idx = 7;   // everything above 5 incl. saturation
  return (sign_bit(v) ? 8u : 0u) | idx;
}

// Stochastic rounding (Sec. 4.4): the value goes to one of its two grid
// neighbours, the upper one with probability (a - lo) / (hi - lo), here
// resolved to 16 bits.  r16 is a uniform integer in [0, 65535].
uint32_t e2m1_encode_sr(float v, uint32_t r16) {
  const float a = std::fabs(v);
  const uint32_t s = sign_bit(v) ? 8u : 0u;
  if (!(a < 6.0f)) return s | 7u;
  uint32_t lo = 0;
  while (lo < 7 && kE2M1Grid[lo + 1] <= a) ++lo;       // grid[lo] <= a < grid[lo+1]
  const float step = kE2M1Grid[lo + 1] - kE2M1Grid[lo];
  const float p = (a - kE2M1Grid[lo]) / step;          // exact: step is a power of two
  const uint32_t T = static_cast<uint32_t>(std::floor(p * 65536.0f));
  const bool up = (T + (r16 & 0xFFFFu)) >= 65536u;
  return s | (up ? lo + 1 : lo);
}

float e4m3_decode(uint32_t code) {
  const uint32_t e = (code >> 3) & 15u, m = code & 7u;
  float mag;
  if (e == 15u && m == 7u) mag = std::numeric_limits<float>::quiet_NaN();
  else if (e == 0u)        mag = std::ldexp(static_cast<float>(m), -9);
  else                     mag = std::ldexp(1.0f + static_cast<float>(m) / 8.0f, static_cast<int>(e) - 7);
  return (code & 0x80u) ? -mag : mag;
}

// Non-negative binary32 -> E4M3 code, round-to-nearest-even, saturating at
// 448 (App. B.2: RNE for the stored decode scale).
uint32_t e4m3_encode_rne_sat(float u) {
  if (!(u > 0.0f)) return 0;
  if (u >= 448.0f) return 0x7E;
  if (u < 0.015625f) {                                  // below 2^-6: fixed step 2^-9
    const float n = std::nearbyint(u * 512.0f);          // exact scaling, ties to even
    return static_cast<uint32_t>(n);                     // 8 lands on the first normal code
  }
  int e;
  std::frexp(u, &e);                                     // u = f * 2^e, f in [0.5, 1)
  e -= 1;                                                // u = 1.xxx * 2^e
  float n = std::nearbyint(std::ldexp(u, 3 - e));        // in [8, 16], ties to even
  if (n == 16.0f) { n = 8.0f; e += 1; }
  return (static_cast<uint32_t>(e + 7) << 3) | (static_cast<uint32_t>(n) - 8u);
}

uint16_t f32_to_bf16_rne(float f) {
  uint32_t w = f32_bits(f);
  if ((w & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((w >> 16) | 0x40u);
  const uint32_t lsb = (w >> 16) & 1u;
  w += 0x7FFFu + lsb;
  return static_cast<uint16_t>(w >> 16);
}

// ---------------------------------------------------------------- Philox4x32-10

void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
    const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    const uint32_t n0 = static_cast<uint32_t>(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = static_cast<uint32_t>(p1);
    const uint32_t n2 = static_cast<uint32_t>(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = static_cast<uint32_t>(p0);
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint32_t sr_random16(uint64_t seed, uint64_t i, uint64_t j) {
  const uint32_t ctr[4] = {static_cast<uint32_t>(j >> 3), static_cast<uint32_t>(i), 0u, 0u};
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  uint32_t w[4];
  philox4x32_10(ctr, key, w);
  const uint32_t e = static_cast<uint32_t>(j & 7u);
  const uint32_t word = w[e >> 1];
  return (e & 1u) ? (word >> 16) : (word & 0xFFFFu);
}

uint32_t rht_sign_mask(uint64_t seed) {
  const uint32_t ctr[4] = {0u, 0u, 0u, 0xFFFFFFFFu};
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  uint32_t w[4];
  philox4x32_10(ctr, key, w);
  return w[0] & 0xFFFFu;
}

// ---------------------------------------------------------------- Hadamard

// In-place unnormalised Walsh-Hadamard butterfly of 16 points, stages
// h = 1, 2, 4, 8, followed by the 1/sqrt(16) normalisation (App. C: H_d is
// the normalised Sylvester matrix).
void hadamard16(float v[16]) {
  for (int h = 1; h < 16; h <<= 1) {
    for (int i = 0; i < 16; ++i) {
      if ((i & h) == 0) {
        const float a = v[i], b = v[i + h];
        v[i] = a + b;
        v[i + h] = a - b;
      }
    }
  }
  for (int i = 0; i < 16; ++i) v[i] = 0.25f * v[i];
}

// y = (v .* s) H_16 : the random sign diagonal multiplies from the left of
// H_d (App. C, H = S_d H_d), so the signs hit the input vector first.
void rht16_forward(float v[16], uint32_t mask) {
  for (int i = 0; i < 16; ++i) if ((mask >> i) & 1u) v[i] = -v[i];
  hadamard16(v);
}

// x = (y H_16^T) .* s ; H_16 is symmetric and H_16 H_16 = I.
void rht16_inverse(float y[16], uint32_t mask) {
  hadamard16(y);
  for (int i = 0; i < 16; ++i) if ((mask >> i) & 1u) y[i] = -y[i];
}

// Other rotation sizes (Sec. 4.2 "Hadamard matrix size", App. E.4: d = 2, 4, 128 are ablated against
// d = 16; d = 32 belongs to the MXFP4 comparison).  Same construction for every d: sign i of the
// diagonal is bit i of the 128 bits the Philox call above returns (word i / 32, bit i % 32), so
// d = 16 gives rht_sign_mask(); butterfly stages h = 1, 2, ..., d / 2 in this order; then one
// multiply by the binary32 nearest to 1 / sqrt(d) (exact for d = 4, 16).
bool rht_dim_ok(int d) { return d == 2 || d == 4 || d == 16 || d == 32 || d == 128; }

void rht_signs(uint64_t seed, int d, uint8_t* negate) {
  const uint32_t ctr[4] = {0u, 0u, 0u, 0xFFFFFFFFu};
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  uint32_t w[4];
  philox4x32_10(ctr, key, w);
  for (int i = 0; i < d; ++i) negate[i] = static_cast<uint8_t>((w[i >> 5] >> (i & 31)) & 1u);
}

void hadamard_d(float* v, int d) {
  for (int h = 1; h < d; h <<= 1)
    for (int i = 0; i < d; ++i)
      if ((i & h) == 0) {
        const float a = v[i], b = v[i + h];
        v[i] = a + b;
        v[i + h] = a - b;
      }
  const float norm = static_cast<float>(1.0 / std::sqrt(static_cast<double>(d)));
  for (int i = 0; i < d; ++i) v[i] = norm * v[i];
}

void rht_forward_d(float* v, int d, const uint8_t* negate) {
  for (int i = 0; i < d; ++i) if (negate[i]) v[i] = -v[i];
  hadamard_d(v, d);
}

void rht_inverse_d(float* y, int d, const uint8_t* negate) {
  hadamard_d(y, d);
  for (int i = 0; i < d; ++i) if (negate[i]) y[i] = -y[i];
}

// ---------------------------------------------------------------- quantize

struct View {            // element (o, k) of the copy's [outer, inner] view
  const uint16_t* x;
  int64_t ld;
  bool transposed;       // false: row copy, true: col copy
  float at(int64_t o, int64_t k) const {
    return bf16_bits_to_f32(transposed ? x[k * ld + o] : x[o * ld + k]);
  }
};

}  // namespace

extern "C" {

float    orc_e2m1_decode(uint32_t code) { return e2m1_decode(code); }
uint32_t orc_e2m1_encode_rne(float v) { return e2m1_encode_rne(v); }
uint32_t orc_e2m1_encode_sr(float v, uint32_t r16) { return e2m1_encode_sr(v, r16); }
float    orc_e4m3_decode(uint32_t code) { return e4m3_decode(code); }
uint32_t orc_e4m3_encode_rne_sat(float u) { return e4m3_encode_rne_sat(u); }
uint32_t orc_f32_to_bf16_rne(float f) { return f32_to_bf16_rne(f); }
void     orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) { philox4x32_10(ctr, key, out); }
uint32_t orc_sr_random16(uint64_t seed, uint64_t i, uint64_t j) { return sr_random16(seed, i, j); }
uint32_t orc_rht_sign_mask(uint64_t seed) { return rht_sign_mask(seed); }
void     orc_rht16_forward(float* v, uint32_t mask) { rht16_forward(v, mask); }
void     orc_rht16_inverse(float* v, uint32_t mask) { rht16_inverse(v, mask); }
int orc_rht_signs(uint64_t seed, int d, uint8_t* negate) {
  if (!rht_dim_ok(d)) return -1;
  rht_signs(seed, d, negate);
  return 0;
}
int orc_rht_forward_d(float* v, int d, const uint8_t* negate) {
  if (!rht_dim_ok(d)) return -1;
  rht_forward_d(v, d, negate);
  return 0;
}
int orc_rht_inverse_d(float* v, int d, const uint8_t* negate) {
  if (!rht_dim_ok(d)) return -1;
  rht_inverse_d(v, d, negate);
  return 0;
}
int      orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// Quantize one copy of a bf16 [rows, cols] tensor (leading dimension ld).
//   copy       0 = row copy (blocks along cols), 1 = col copy (blocks along
//              rows, stored transposed)
//   block_dim  1 = 1x16 blocks, 16 = 16x16 blocks (weights, Sec. 4.3)
//   rounding   0 = round-to-nearest-even, 1 = stochastic
//   rht_dim    0, or the size d of the rotation: each aligned group of d along
//              the block direction is rotated before anything else (Wgrad
//              operands, Sec. 4.2; d = 16 is the paper's choice)
//   amax_given null, or the amax to use in Eq. 1 instead of this tensor's own
//              (in the rotated space for a rotated copy)
// Outputs: codes [outer, inner/2] bytes, scales [outer, inner/16] bytes,
// tensor_scale[0] = s_dec, tensor_scale[1] = amax (in the rotated space for a
// rotated copy).  Returns 0, or -1 for bad arguments.
// per_row: one tensor-level scale per row of the copy ([outer] of them) instead of one per tensor;
// tensor_scale then receives s_dec[0 .. outer) followed by amax[0 .. outer).
static int quantize_impl(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld,
                 int copy, int block_dim, int rounding, int rht_dim,
                 uint64_t rht_seed, uint64_t sr_seed, const float* amax_given, bool per_row,
                 uint8_t* codes, uint8_t* scales, float* tensor_scale) {
  if (!x || !codes || !scales || !tensor_scale) return -1;
  if (per_row && (block_dim != 1 || amax_given)) return -1;
  if (rows < 0 || cols < 0 || ld < cols) return -1;
  if (copy != 0 && copy != 1) return -1;
  if (block_dim != 1 && block_dim != 16) return -1;
  if ((copy == 0 ? cols : rows) % 16) return -1;             // whole blocks along the block direction
  if (block_dim == 16 && (rows % 16 || cols % 16)) return -1;
  if (block_dim == 16 && rht_dim) return -1;   // the paper never rotates weights (Sec. 4.3)
  if (rht_dim && (!rht_dim_ok(rht_dim) || (copy == 0 ? cols : rows) % rht_dim)) return -1;

  const View view{x, ld, copy == 1};
  const int64_t outer = copy == 1 ? cols : rows;
  const int64_t inner = copy == 1 ? rows : cols;
  const int64_t nblk = inner / 16;
  uint8_t negate[128] = {0};
  if (rht_dim) rht_signs(rht_seed, rht_dim, negate);

  // Step 0: the values to be quantized, in binary32, rotated if asked.
  std::vector<float> w(static_cast<size_t>(outer) * static_cast<size_t>(inner));
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < outer; ++o) {
    float* wo = w.data() + o * inner;
    for (int64_t k = 0; k < inner; ++k) wo[k] = view.at(o, k);
    if (rht_dim)
      for (int64_t g = 0; g < inner / rht_dim; ++g) rht_forward_d(wo + rht_dim * g, rht_dim, negate);
  }

  // App. B.1, Eq. 1: tensor-level scale from the global amax -- of this tensor, or one the caller supplies
  // (an amax known beforehand or reduced over the shards of a larger tensor saves the first of the two passes
  // over memory that App. B.1 counts; nothing else changes, values beyond it saturate as in Eq. 3-4).
  // With per_row the same equation is evaluated once per row of the copy, with that row's amax (App. B.1, last
  // sentence): s_enc_of[o], s_dec_of[o] are the scales row o is quantized with in either mode.
  auto eq1 = [](float amax, float& s_enc, float& s_dec) {
    if (amax == 0.0f) {
      s_enc = 1.0f;                                  // all-zero tensor: any scale encodes it
    } else {
      s_enc = (6.0f * 448.0f) / amax;
      if (std::isinf(s_enc)) s_enc = std::numeric_limits<float>::max();
    }
    s_dec = 1.0f / s_enc;
  };
  std::vector<float> s_enc_of(static_cast<size_t>(outer)), s_dec_of(static_cast<size_t>(outer));
  if (!per_row) {
    float amax = 0.0f;
    if (amax_given) {
      amax = *amax_given;
      if (!(amax >= 0.0f)) return -1;
    } else {
      for (size_t t = 0; t < w.size(); ++t) {
        const float a = std::fabs(w[t]);
        if (a > amax) amax = a;
      }
    }
    float s_enc, s_dec;
    eq1(amax, s_enc, s_dec);
    tensor_scale[0] = s_dec;
    tensor_scale[1] = amax;
    for (int64_t o = 0; o < outer; ++o) {
      s_enc_of[o] = s_enc;
      s_dec_of[o] = s_dec;
    }
  } else {
    for (int64_t o = 0; o < outer; ++o) {
      float amax = 0.0f;
      for (int64_t k = 0; k < inner; ++k) {
        const float a = std::fabs(w[o * inner + k]);
        if (a > amax) amax = a;
      }
      eq1(amax, s_enc_of[o], s_dec_of[o]);
      tensor_scale[o] = s_dec_of[o];
      tensor_scale[outer + o] = amax;
    }
  }

  // App. B.2, Eq. 2-3: per-block decode scale, stored as E4M3.
  // For 16x16 blocks the amax runs over the tile and every 1x16 slice of the
  // tile gets the same stored scale (Sec. 4.3).
  std::vector<float> blk_amax(static_cast<size_t>(outer) * static_cast<size_t>(nblk));
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < outer; ++o)
    for (int64_t b = 0; b < nblk; ++b) {
      float m = 0.0f;
      for (int k = 0; k < 16; ++k) {
        const float a = std::fabs(w[o * inner + 16 * b + k]);
        if (a > m) m = a;
      }
      blk_amax[o * nblk + b] = m;
    }
  if (block_dim == 16) {
    for (int64_t ot = 0; ot < outer / 16; ++ot)
      for (int64_t b = 0; b < nblk; ++b) {
        float m = 0.0f;
        for (int r = 0; r < 16; ++r) {
          const float a = blk_amax[(16 * ot + r) * nblk + b];
          if (a > m) m = a;
        }
        for (int r = 0; r < 16; ++r) blk_amax[(16 * ot + r) * nblk + b] = m;
      }
  }

#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < outer; ++o) {
    const float s_enc = s_enc_of[o], s_dec = s_dec_of[o];
    for (int64_t b = 0; b < nblk; ++b) {
      const float s_dec_b = blk_amax[o * nblk + b] / 6.0f;          // Eq. 2
      const uint32_t sc = e4m3_encode_rne_sat(s_dec_b * s_enc);     // Eq. 3
      scales[o * nblk + b] = static_cast<uint8_t>(sc);
      const float sd = e4m3_decode(sc);
      // "real" local encode scale: invert the stored scale in binary32 and
      // bring it back to the tensor's range (App. B.2).
      const float denom = sd * s_dec;
      const float s_enc_b = (denom == 0.0f) ? 0.0f : 1.0f / denom;
      for (int k = 0; k < 16; k += 2) {
        uint32_t c[2];
        for (int t = 0; t < 2; ++t) {
          const int64_t kk = 16 * b + k + t;
          const float v = w[o * inner + kk] * s_enc_b;               // Eq. 4
          if (rounding == 0) {
            c[t] = e2m1_encode_rne(v);
          } else {
            const uint64_t li = (copy == 1) ? static_cast<uint64_t>(kk) : static_cast<uint64_t>(o);
            const uint64_t lj = (copy == 1) ? static_cast<uint64_t>(o) : static_cast<uint64_t>(kk);
            c[t] = e2m1_encode_sr(v, sr_random16(sr_seed, li, lj));
          }
        }
        codes[o * (inner / 2) + (16 * b + k) / 2] = static_cast<uint8_t>(c[0] | (c[1] << 4));
      }
    }
  }
  return 0;
}

int orc_quantize(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld,
                 int copy, int block_dim, int rounding, int rht_dim,
                 uint64_t rht_seed, uint64_t sr_seed, const float* amax_given,
                 uint8_t* codes, uint8_t* scales, float* tensor_scale) {
  return quantize_impl(x, rows, cols, ld, copy, block_dim, rounding, rht_dim, rht_seed, sr_seed, amax_given, false,
                       codes, scales, tensor_scale);
}

// The same with one tensor-level scale per row of the copy (App. B.1, last sentence): 1x16 blocks only;
// tensor_scale: float[2 * outer] = s_dec of every row, then the amax of every row.
int orc_quantize_row_scales(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld,
                            int copy, int rounding, int rht_dim, uint64_t rht_seed, uint64_t sr_seed,
                            uint8_t* codes, uint8_t* scales, float* tensor_scale) {
  return quantize_impl(x, rows, cols, ld, copy, 1, rounding, rht_dim, rht_seed, sr_seed, nullptr, true,
                       codes, scales, tensor_scale);
}

// Decode a quantized copy [outer, inner] back to binary32:
// value(code) * fp32(stored block scale), then * s_dec (Sec. 2: decode with
// the reciprocal of the encode scale; App. B.2).  With undo_rht_dim = d each
// aligned group of d is rotated back.
int orc_dequantize(const uint8_t* codes, const uint8_t* scales, float s_dec,
                   int64_t outer, int64_t inner, int undo_rht_dim, uint64_t rht_seed,
                   float* out) {
  if (!codes || !scales || !out || inner % 16) return -1;
  if (undo_rht_dim && (!rht_dim_ok(undo_rht_dim) || inner % undo_rht_dim)) return -1;
  uint8_t negate[128] = {0};
  if (undo_rht_dim) rht_signs(rht_seed, undo_rht_dim, negate);
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < outer; ++o) {
    float* row = out + o * inner;
    for (int64_t k = 0; k < inner; ++k) {
      const float sd = e4m3_decode(scales[o * (inner / 16) + k / 16]);
      const uint8_t byte = codes[o * (inner / 2) + k / 2];
      const uint32_t c = (k & 1) ? (byte >> 4) : (byte & 15u);
      const float t = e2m1_decode(c) * sd;
      row[k] = t * s_dec;
    }
    if (undo_rht_dim)
      for (int64_t g = 0; g < inner / undo_rht_dim; ++g) rht_inverse_d(row + undo_rht_dim * g, undo_rht_dim, negate);
  }
  return 0;
}

static inline double deq_f64(const uint8_t* codes, const uint8_t* scales, double s_dec,
                             int64_t K, int64_t o, int64_t k) {
  const uint8_t byte = codes[o * (K / 2) + k / 2];
  const uint32_t c = (k & 1) ? (byte >> 4) : (byte & 15u);
  return static_cast<double>(e2m1_decode(c)) *
         static_cast<double>(e4m3_decode(scales[o * (K / 16) + k / 16])) * s_dec;
}

// Reference GEMM in binary64 on the dequantized operands:
// D[m, n] = sum_k A[m, k] * B[n, k], both operands [outer, K] quantized copies.
int orc_gemm_f64(const uint8_t* a_codes, const uint8_t* a_scales, float a_sdec,
                 const uint8_t* b_codes, const uint8_t* b_scales, float b_sdec,
                 int64_t M, int64_t N, int64_t K, double* D) {
  if (K % 16) return -1;
  std::vector<double> A(static_cast<size_t>(M) * K), B(static_cast<size_t>(N) * K);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t k = 0; k < K; ++k) A[m * K + k] = deq_f64(a_codes, a_scales, a_sdec, K, m, k);
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t k = 0; k < K; ++k) B[n * K + k] = deq_f64(b_codes, b_scales, b_sdec, K, n, k);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double acc = 0.0;
      for (int64_t k = 0; k < K; ++k) acc += A[m * K + k] * B[n * K + k];
      D[m * N + n] = acc;
    }
  return 0;
}

// The same reference for a list of output entries (m_idx[t], n_idx[t]).
int orc_gemm_f64_entries(const uint8_t* a_codes, const uint8_t* a_scales, float a_sdec,
                         const uint8_t* b_codes, const uint8_t* b_scales, float b_sdec,
                         int64_t K, int64_t count, const int64_t* m_idx, const int64_t* n_idx,
                         double* out) {
  if (K % 16) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < count; ++t) {
    double acc = 0.0;
    for (int64_t k = 0; k < K; ++k)
      acc += deq_f64(a_codes, a_scales, a_sdec, K, m_idx[t], k) *
             deq_f64(b_codes, b_scales, b_sdec, K, n_idx[t], k);
    out[t] = acc;
  }
  return 0;
}

// Decode, and the binary64 reference GEMM, for copies whose tensor-level scale is per row of the copy (App. B.1,
// last sentence).  a_sdec / b_sdec point to one decode scale per row when the per-row flag of that operand is
// set, to a single one otherwise (so a per-row activation meets a per-tensor weight).  Eq. 5's two tensor-level
// factors become s_dec^A[m] * s_dec^B[n]: still constant along k, which is what lets them stay outside the sum.
int orc_dequantize_row_scales(const uint8_t* codes, const uint8_t* scales, const float* s_dec,
                              int64_t outer, int64_t inner, int undo_rht_dim, uint64_t rht_seed, float* out) {
  if (!codes || !scales || !s_dec || !out || inner % 16) return -1;
  if (undo_rht_dim && (!rht_dim_ok(undo_rht_dim) || inner % undo_rht_dim)) return -1;
  uint8_t negate[128] = {0};
  if (undo_rht_dim) rht_signs(rht_seed, undo_rht_dim, negate);
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < outer; ++o) {
    float* row = out + o * inner;
    for (int64_t k = 0; k < inner; ++k) {
      const float sd = e4m3_decode(scales[o * (inner / 16) + k / 16]);
      const uint8_t byte = codes[o * (inner / 2) + k / 2];
      const uint32_t c = (k & 1) ? (byte >> 4) : (byte & 15u);
      const float t = e2m1_decode(c) * sd;
      row[k] = t * s_dec[o];
    }
    if (undo_rht_dim)
      for (int64_t g = 0; g < inner / undo_rht_dim; ++g) rht_inverse_d(row + undo_rht_dim * g, undo_rht_dim, negate);
  }
  return 0;
}

int orc_gemm_f64_row_scales(const uint8_t* a_codes, const uint8_t* a_scales, const float* a_sdec, int a_per_row,
                            const uint8_t* b_codes, const uint8_t* b_scales, const float* b_sdec, int b_per_row,
                            int64_t M, int64_t N, int64_t K, double* D) {
  if (K % 16 || !a_sdec || !b_sdec) return -1;
  std::vector<double> A(static_cast<size_t>(M) * K), B(static_cast<size_t>(N) * K);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t k = 0; k < K; ++k) A[m * K + k] = deq_f64(a_codes, a_scales, a_sdec[a_per_row ? m : 0], K, m, k);
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t k = 0; k < K; ++k) B[n * K + k] = deq_f64(b_codes, b_scales, b_sdec[b_per_row ? n : 0], K, n, k);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double acc = 0.0;
      for (int64_t k = 0; k < K; ++k) acc += A[m * K + k] * B[n * K + k];
      D[m * N + n] = acc;
    }
  return 0;
}

// Eq. 5 as written: per 16-block, the partial dot product of the FP4 values
// times both stored block scales, accumulated in binary32 in block order; the
// two tensor-level decode scales are applied to the finished sum.
int orc_gemm_f32_blockscaled(const uint8_t* a_codes, const uint8_t* a_scales, float a_sdec,
                             const uint8_t* b_codes, const uint8_t* b_scales, float b_sdec,
                             int64_t M, int64_t N, int64_t K, float* D) {
  if (K % 16) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      float acc = 0.0f;
      for (int64_t b = 0; b < K / 16; ++b) {
        float partial = 0.0f;
        for (int k = 0; k < 16; ++k) {
          const int64_t kk = 16 * b + k;
          const uint8_t ab = a_codes[m * (K / 2) + kk / 2], bb = b_codes[n * (K / 2) + kk / 2];
          const float av = e2m1_decode((kk & 1) ? (ab >> 4) : (ab & 15u));
          const float bv = e2m1_decode((kk & 1) ? (bb >> 4) : (bb & 15u));
          partial += av * bv;
        }
        const float sa = e4m3_decode(a_scales[m * (K / 16) + b]);
        const float sb = e4m3_decode(b_scales[n * (K / 16) + b]);
        acc += (sa * sb) * partial;
      }
      D[m * N + n] = acc * (a_sdec * b_sdec);
    }
  return 0;
}


// ======================================================================
// MXFP4, the comparison format (Sec. 2 second and third paragraphs; App. B.4
// "Remarks on MXFP4 and NVFP4 scale factor"; Sec. 5 for its 32-point rotation).
//   * blocks of 32 consecutive elements along the copy's contiguous dimension
//   * one unsigned E8M0 scale per block: a power of two 2^e, stored as e + 127
//   * the scale is amax_b / 6 rounded UP to the next power of two (App. B.4:
//     decode scales are rounded up so that nothing saturates); no tensor scale
//   * elements are E2M1 codes of x / 2^e, same rounding rules as above
//   * Wgrad operands are rotated with a 32-point transform (Sec. 5)
// Conventions fixed here: amax_b / 6 is one binary32 division; an all-zero
// block stores e = -127; e is clamped to [-127, 127]; the 32-point transform
// is y = H32 (s .* v), butterfly stages h = 1, 2, 4, 8, 16, then one multiply
// by fl(1/sqrt(32)); its sign vector is all 32 bits of word 0 of the Philox
// call that gives the 16-point mask; stochastic rounding of the row copy
// uses the draws above, the col copy draws its own: element (i, j) of the
// logical tensor uses counter (i / 8, j, 1, 0), word (i % 8) / 2, low half
// for even i (eight consecutive rows of a column share one call).
// ======================================================================

namespace {

const float kInvSqrt32 = 0.176776695296636893f;   // nearest binary32 to 1/sqrt(32)

uint32_t rht_sign_mask32(uint64_t seed) {
  const uint32_t ctr[4] = {0u, 0u, 0u, 0xFFFFFFFFu};
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  uint32_t w[4];
  philox4x32_10(ctr, key, w);
  return w[0];
}

void hadamard32(float v[32]) {
  for (int h = 1; h < 32; h <<= 1)
    for (int i = 0; i < 32; ++i)
      if ((i & h) == 0) {
        const float a = v[i], b = v[i + h];
        v[i] = a + b;
        v[i + h] = a - b;
      }
  for (int i = 0; i < 32; ++i) v[i] = kInvSqrt32 * v[i];
}

void rht32_forward(float v[32], uint32_t mask) {
  for (int i = 0; i < 32; ++i) if ((mask >> i) & 1u) v[i] = -v[i];
  hadamard32(v);
}

void rht32_inverse(float y[32], uint32_t mask) {
  hadamard32(y);
  for (int i = 0; i < 32; ++i) if ((mask >> i) & 1u) y[i] = -y[i];
}

// smallest e with 2^e >= s (s >= 0), clamped to the UE8M0 range
int ue8m0_exponent_round_up(float s) {
  if (!(s > 0.0f)) return -127;
  int ex;
  const float m = std::frexp(s, &ex);        // s = m * 2^ex, 0.5 <= m < 1
  int e = (m == 0.5f) ? ex - 1 : ex;
  if (e < -127) e = -127;
  if (e > 127) e = 127;
  return e;
}

uint32_t mx_col_random16(uint64_t seed, uint64_t i, uint64_t j) {
  const uint32_t ctr[4] = {static_cast<uint32_t>(i >> 3), static_cast<uint32_t>(j), 1u, 0u};
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  uint32_t w[4];
  philox4x32_10(ctr, key, w);
  const uint32_t e = static_cast<uint32_t>(i & 7u);
  const uint32_t word = w[e >> 1];
  return (e & 1u) ? (word >> 16) : (word & 0xFFFFu);
}

inline double mx_deq_f64(const uint8_t* codes, const uint8_t* scales, int64_t K, int64_t o, int64_t k) {
  const uint8_t byte = codes[o * (K / 2) + k / 2];
  const uint32_t c = (k & 1) ? (byte >> 4) : (byte & 15u);
  return std::ldexp(static_cast<double>(e2m1_decode(c)), static_cast<int>(scales[o * (K / 32) + k / 32]) - 127);
}

}  // namespace

uint32_t orc_rht_sign_mask32(uint64_t seed) { return rht_sign_mask32(seed); }
void     orc_rht32_forward(float* v, uint32_t mask) { rht32_forward(v, mask); }
void     orc_rht32_inverse(float* v, uint32_t mask) { rht32_inverse(v, mask); }
int      orc_ue8m0_exponent_round_up(float s) { return ue8m0_exponent_round_up(s); }
uint32_t orc_mx_col_random16(uint64_t seed, uint64_t i, uint64_t j) { return mx_col_random16(seed, i, j); }

// Quantize one copy of a bf16 [rows, cols] tensor to MXFP4.  Arguments as for
// orc_quantize; scales [outer, inner/32] UE8M0 bytes; amax_out (may be null)
// receives the largest magnitude seen (rotated space for a rotated copy).
int orc_mx_quantize(const uint16_t* x, int64_t rows, int64_t cols, int64_t ld, int copy, int rounding,
                    int use_rht, uint64_t rht_seed, uint64_t sr_seed, uint8_t* codes, uint8_t* scales,
                    float* amax_out) {
  if (!x || !codes || !scales) return -1;
  if (rows < 0 || cols < 0 || ld < cols) return -1;
  if (copy != 0 && copy != 1) return -1;
  if ((copy == 0 ? cols : rows) % 32) return -1;
  const View view{x, ld, copy == 1};
  const int64_t outer = copy == 1 ? cols : rows;
  const int64_t inner = copy == 1 ? rows : cols;
  const int64_t nblk = inner / 32;
  const uint32_t mask = use_rht ? rht_sign_mask32(rht_seed) : 0u;
  float amax_all = 0.0f;
#pragma omp parallel for schedule(static) reduction(max : amax_all)
  for (int64_t o = 0; o < outer; ++o) {
    for (int64_t b = 0; b < nblk; ++b) {
      float w[32];
      for (int k = 0; k < 32; ++k) w[k] = view.at(o, 32 * b + k);
      if (use_rht) rht32_forward(w, mask);
      float amax_b = 0.0f;
      for (int k = 0; k < 32; ++k) {
        const float a = std::fabs(w[k]);
        if (a > amax_b) amax_b = a;
      }
      if (amax_b > amax_all) amax_all = amax_b;
      const int e = ue8m0_exponent_round_up(amax_b / 6.0f);
      scales[o * nblk + b] = static_cast<uint8_t>(e + 127);
      const float inv = std::ldexp(1.0f, -e);              // 2^-e, exact (subnormal for e = 127)
      for (int k = 0; k < 32; k += 2) {
        uint32_t c[2];
        for (int t = 0; t < 2; ++t) {
          const int64_t kk = 32 * b + k + t;
          const float v = w[k + t] * inv;
          if (rounding == 0) {
            c[t] = e2m1_encode_rne(v);
          } else if (copy == 0) {
            c[t] = e2m1_encode_sr(v, sr_random16(sr_seed, static_cast<uint64_t>(o), static_cast<uint64_t>(kk)));
          } else {
            c[t] = e2m1_encode_sr(v, mx_col_random16(sr_seed, static_cast<uint64_t>(kk), static_cast<uint64_t>(o)));
          }
        }
        codes[o * (inner / 2) + (32 * b + k) / 2] = static_cast<uint8_t>(c[0] | (c[1] << 4));
      }
    }
  }
  if (amax_out) *amax_out = amax_all;
  return 0;
}

int orc_mx_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t outer, int64_t inner, int undo_rht,
                      uint64_t rht_seed, float* out) {
  if (!codes || !scales || !out || inner % 32) return -1;
  const uint32_t mask = undo_rht ? rht_sign_mask32(rht_seed) : 0u;
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < outer; ++o)
    for (int64_t b = 0; b < inner / 32; ++b) {
      const int e = static_cast<int>(scales[o * (inner / 32) + b]) - 127;
      float g[32];
      for (int k = 0; k < 32; ++k) {
        const uint8_t byte = codes[o * (inner / 2) + (32 * b + k) / 2];
        g[k] = std::ldexp(e2m1_decode((k & 1) ? (byte >> 4) : (byte & 15u)), e);
      }
      if (undo_rht) rht32_inverse(g, mask);
      for (int k = 0; k < 32; ++k) out[o * inner + 32 * b + k] = g[k];
    }
  return 0;
}

// binary64 reference GEMM on MXFP4 operands, whole matrix or listed entries
int orc_mx_gemm_f64(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes, const uint8_t* b_scales,
                    int64_t M, int64_t N, int64_t K, double* D) {
  if (K % 32) return -1;
  std::vector<double> A(static_cast<size_t>(M) * K), B(static_cast<size_t>(N) * K);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t k = 0; k < K; ++k) A[m * K + k] = mx_deq_f64(a_codes, a_scales, K, m, k);
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t k = 0; k < K; ++k) B[n * K + k] = mx_deq_f64(b_codes, b_scales, K, n, k);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double acc = 0.0;
      for (int64_t k = 0; k < K; ++k) acc += A[m * K + k] * B[n * K + k];
      D[m * N + n] = acc;
    }
  return 0;
}

int orc_mx_gemm_f64_entries(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                            const uint8_t* b_scales, int64_t K, int64_t count, const int64_t* m_idx,
                            const int64_t* n_idx, double* out) {
  if (K % 32) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < count; ++t) {
    double acc = 0.0;
    for (int64_t k = 0; k < K; ++k)
      acc += mx_deq_f64(a_codes, a_scales, K, m_idx[t], k) * mx_deq_f64(b_codes, b_scales, K, n_idx[t], k);
    out[t] = acc;
  }
  return 0;
}

}  // extern "C"
