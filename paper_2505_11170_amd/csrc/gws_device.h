// Device-side building blocks of the GaussWS kernels (gfx950 only).
// Internal to csrc/: not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gws {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): the counter-based bit source named in
// the paper's Sec. 3.4.  One call yields the 128 bits of a group of 8
// row-contiguous elements (16 bits per element).
// ---------------------------------------------------------------------------
struct Philox4 {
  uint32_t x0, x1, x2, x3;
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Philox4{c0, c1, c2, c3};
}

// ---------------------------------------------------------------------------
// 128 random bits -> eight 4-bit sign-magnitude codes of R (paper Sec. 3.4,
// Eq. 9 and Eq. 10), evaluated for all eight elements at once: element k owns
// nibble k of each word.
//   |R| = 2 : (b|b) & (8 bits all set)                 -> 3/4 * 2^-8
//   |R| = 1 : (b|b) & (b|b) & b, unless |R| = 2        -> (3/4)^2 * 2^-1 * (1 - P(|R|=2))
//   sign    : 1 bit
// code = sign<<3 | |R|, element k in bits 4k..4k+3.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t noise_codes(const Philox4& x) {
  uint32_t all8 = x.x0 & x.x1;      // per nibble: AND of the 8 bits, folded below
  all8 &= all8 >> 1;
  all8 &= all8 >> 2;                // bit 0 of each nibble = all 8 bits set
  const uint32_t v = x.x2 | (x.x2 >> 1);  // bit 0: b|b (A), bit 2: b|b (C)
  const uint32_t y = x.x3 | (x.x3 >> 1);  // bit 0: b|b (D)
  const uint32_t m2 = all8 & v & 0x11111111u;
  const uint32_t m1 = (v >> 2) & y & (x.x3 >> 2) & ~m2 & 0x11111111u;
  return (x.x3 & 0x88888888u) | (m2 << 1) | m1;
}

__device__ __forceinline__ uint32_t group_codes(uint32_t cg, uint32_t row, uint32_t step_lo,
                                                uint32_t step_hi, uint32_t seed_lo, uint32_t seed_hi) {
  return noise_codes(philox4x32_10(cg, row, step_lo, step_hi, seed_lo, seed_hi));
}

// ---------------------------------------------------------------------------
// 2^t as one fixed fp32 function (for the block scale 2^(1-b_t) of Eq. 3 with a
// real-valued b_t): n = rint(t), f = t - n, degree-6 Horner polynomial in f with
// fused multiply-adds, scaled by 2^n.  Exact for integer t.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float exp2_fixed(float t) {
  const float n = rintf(t);
  const float f = t - n;
  float p = __uint_as_float(0x39222002u);
  p = __fmaf_rn(p, f, __uint_as_float(0x3AAF844Bu));
  p = __fmaf_rn(p, f, __uint_as_float(0x3C1D950Eu));
  p = __fmaf_rn(p, f, __uint_as_float(0x3D6357B6u));
  p = __fmaf_rn(p, f, __uint_as_float(0x3E75FDF0u));
  p = __fmaf_rn(p, f, __uint_as_float(0x3F317218u));
  p = __fmaf_rn(p, f, 1.0f);
  return ldexpf(p, (int)n);
}

// fp32 -> BF16 bits, round to nearest even (finite values).
__device__ __forceinline__ uint32_t bf16_rne_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// ---------------------------------------------------------------------------
// Per-block constants of the forward pass.
// ---------------------------------------------------------------------------
struct BlockScale {
  float s32;        // max|w| * 2^(1-b_t), unrounded fp32 (stored; Eq. 4 reuses it)
  float s;          // bf16_rne(s32) as fp32: the step of the PQN
  uint32_t emin_b;  // cast: fp32 exponent field (<<23) of the lowest normal binade of X*format
  uint32_t max_b;   // cast: fp32 bits of max*X (saturation bound)
};

template <int EMAX, int EMIN>
__device__ __forceinline__ void cast_constants(uint32_t a16, BlockScale& b) {
  // Ea = floor(log2 max|w|) from the BF16 exponent field; clamped so that every
  // constant below is a normal fp32 (blocks with max|w| < 2^-100 are outside the
  // supported domain and only have to stay in bounds).
  int ef = (int)(a16 >> 7);
  ef = ef < 27 ? 27 : ef;
  b.emin_b = (uint32_t)(ef + 1 - EMAX + EMIN) << 23;  // X = 2^(Ea+1-EMAX), lowest normal = X * 2^EMIN
  b.max_b = ((uint32_t)(ef + 1) << 23) | 0x00600000u; // 1.75 * 2^EMAX * X = 1.75 * 2^(Ea+1)
}

__device__ __forceinline__ BlockScale block_scale(uint32_t a16, float bt) {
  BlockScale b;
  const float a = __uint_as_float(a16 << 16);
  const float p = exp2_fixed(1.0f - bt);
  b.s32 = a * p;
  b.s = __uint_as_float(bf16_rne_bits(b.s32) << 16);
  b.emin_b = 0;
  b.max_b = 0;
  return b;
}

// ---------------------------------------------------------------------------
// Block-scaled fp_{e,m} cast (paper Sec. 3.3) of a BF16 value held in fp32:
// round to nearest even onto the grid of spacing 2^(max(e_v, emin) - M), by
// adding and subtracting 2^(23 - M) times that binade (the fp32 adder performs
// the rounding), then saturate and restore the sign.
// ---------------------------------------------------------------------------
template <int M>
__device__ __forceinline__ float cast_scaled(float v, const BlockScale& b) {
  const uint32_t u = __float_as_uint(v);
  const uint32_t au = u & 0x7FFFFFFFu;
  uint32_t eb = au & 0x7F800000u;
  eb = eb > b.emin_b ? eb : b.emin_b;
  const float c = __uint_as_float(eb + ((uint32_t)(23 - M) << 23));
  float r = (__uint_as_float(au) + c) - c;
  r = fminf(r, __uint_as_float(b.max_b));
  return __uint_as_float(__float_as_uint(r) | (u & 0x80000000u));
}

// One element of Eq. 3 + cast: w (BF16 value in fp32), its 4-bit noise code and
// the block constants -> BF16 bits of w_hat.
template <int FMT>
__device__ __forceinline__ uint32_t sample_element(float w, uint32_t code, const BlockScale& b) {
  // PQN = R * s in sign-magnitude: |R| * s is exact, the sign bit is placed as is
  const float mag = (float)(code & 3u);
  const float pqn = __uint_as_float(__float_as_uint(mag * b.s) | ((code & 8u) << 28));
  const float sum = w + pqn;  // fp32 add, then one RNE to BF16 == exact BF16 add
  const uint32_t h = bf16_rne_bits(sum);
  if (FMT == 0) return h;
  const float v = __uint_as_float(h << 16);
  const float q = (FMT == 1) ? cast_scaled<3>(v, b) : cast_scaled<2>(v, b);
  return __float_as_uint(q) >> 16;
}

// Max / sum over the 32 lanes of a wavefront that share a 32x32 block.  Lane =
// 8 * row_in_8 + column_group; a block owns column groups {0..3} or {4..7}, so
// the lanes of one block differ in lane bits 0, 1, 3, 4, 5.
__device__ __forceinline__ uint32_t block_max_u32(uint32_t v) {
  v = max(v, (uint32_t)__shfl_xor((int)v, 1));
  v = max(v, (uint32_t)__shfl_xor((int)v, 2));
  v = max(v, (uint32_t)__shfl_xor((int)v, 8));
  v = max(v, (uint32_t)__shfl_xor((int)v, 16));
  v = max(v, (uint32_t)__shfl_xor((int)v, 32));
  return v;
}

__device__ __forceinline__ float block_sum_f32(float v) {
  v += __shfl_xor(v, 1);
  v += __shfl_xor(v, 2);
  v += __shfl_xor(v, 8);
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

}  // namespace gws
