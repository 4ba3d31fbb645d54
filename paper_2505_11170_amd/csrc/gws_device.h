// Device-side building blocks of the GaussWS kernels (gfx950 only).
// Internal to csrc/: not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gws {

// Pointers into global memory, typed as such: the accesses through them are global (not
// flat) instructions whatever the pointer's provenance.
#define GWS_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ GWS_GLOBAL T* global_ptr(const void* p) {
  return (GWS_GLOBAL T*)(uintptr_t)p;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): the counter-based bit source named in
// the paper's Sec. 3.4.  One call yields the 128 bits of a group of 8
// row-contiguous elements (16 bits per element).  Counter = (column group,
// row, step lo, step hi), key = per-tensor seed.  Calls of one lane that differ
// only in the row share the multiplies of the first rounds (the compiler folds
// them once the calls are inlined side by side).
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
    const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
    const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Philox4{c0, c1, c2, c3};
}

// The four Philox calls of a lane (rows row[0..3], one column group) with the work of the first three rounds
// that does not depend on all of the counter done once.  With counter (cg, row, step_lo, step_hi):
//   round 0: M1 * step_lo is uniform; M0 * cg depends on the column group only; the new c0 on the row only;
//   round 1: M0 * c0 depends on the row only (PhiloxRows: kept across the column tiles a wavefront walks),
//            M1 * c2 on the column group only;
//   round 2: M0 * c0 depends on the column group only; from M1 * c2 on everything depends on both.
// 63 multiplies per four calls instead of 80 (67 with the row part), same bits as philox4x32_10:
// philox_rows once per wavefront, philox_cols once per tile, philox_row per call.
struct PhiloxRows {
  uint32_t hi[4], lo[4];   // M0 * (c0 after round 0) for the four rows
};

__device__ __forceinline__ PhiloxRows philox_rows(const uint32_t (&row)[4], uint32_t step_lo, uint32_t k0) {
  const uint32_t base = (uint32_t)(((uint64_t)0xCD9E8D57u * step_lo) >> 32) ^ k0;   // uniform
  PhiloxRows r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint64_t d = (uint64_t)0xD2511F53u * (base ^ row[i]);
    r.hi[i] = (uint32_t)(d >> 32);
    r.lo[i] = (uint32_t)d;
  }
  return r;
}

// The column-group share of the first three rounds (four registers), then one call per row.
struct PhiloxCols {
  uint32_t c3_1, c1_2, hi_f, c3_3;
};

__device__ __forceinline__ PhiloxCols philox_cols(uint32_t cg, uint32_t step_lo, uint32_t step_hi, uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u;
  const uint32_t c1_1 = (uint32_t)((uint64_t)M1 * step_lo);                      // round 0, uniform
  const uint64_t b = (uint64_t)M0 * cg;                                          // round 0, column group
  const uint32_t c2_1 = xor3((uint32_t)(b >> 32), step_hi, k1);
  const uint64_t c = (uint64_t)M1 * c2_1;                                        // round 1, column group
  const uint32_t c0_2 = xor3((uint32_t)(c >> 32), c1_1, k0 + W0);
  const uint64_t f = (uint64_t)M0 * c0_2;                                        // round 2, column group
  return PhiloxCols{(uint32_t)b, (uint32_t)c, (uint32_t)(f >> 32), (uint32_t)f};
}

// Call i of the four: the row share joins in round 1.
__device__ __forceinline__ Philox4 philox_row(const PhiloxCols& pc, const PhiloxRows& rp, int i, uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  const uint32_t c2_2 = xor3(rp.hi[i], pc.c3_1, k1 + W1), c3_2 = rp.lo[i];       // round 1
  const uint64_t e = (uint64_t)M1 * c2_2;                                        // round 2
  uint32_t c0 = xor3((uint32_t)(e >> 32), pc.c1_2, k0 + 2 * W0), c1 = (uint32_t)e;
  uint32_t c2 = xor3(pc.hi_f, c3_2, k1 + 2 * W1), c3 = pc.c3_3;
  uint32_t ka = k0 + 3 * W0, kb = k1 + 3 * W1;
#pragma unroll
  for (int r = 3; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)M0 * c0, p1 = (uint64_t)M1 * c2;
    const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, ka), n2 = xor3((uint32_t)(p0 >> 32), c3, kb);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    ka += W0;
    kb += W1;
  }
  return Philox4{c0, c1, c2, c3};
}

// The calls of two tiles (column groups pc[0], pc[1]; the same four rows) advanced round by round together: for a
// wavefront that has its SIMD to itself this is what keeps the vector ALU fed (sixteen independent multiplies per
// round instead of two dependent chains).
__device__ __forceinline__ void philox_two_tiles(const PhiloxCols (&pc)[2], const PhiloxRows& rp, uint32_t k0, uint32_t k1,
                                                 Philox4 (&out)[2][4]) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0[8], c1[8], c2[8], c3[8];
  uint64_t e[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) e[k] = (uint64_t)M1 * xor3(rp.hi[k & 3], pc[k >> 2].c3_1, k1 + W1);   // rounds 1 and 2
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    c0[k] = xor3((uint32_t)(e[k] >> 32), pc[k >> 2].c1_2, k0 + 2 * W0);
    c1[k] = (uint32_t)e[k];
    c2[k] = xor3(pc[k >> 2].hi_f, rp.lo[k & 3], k1 + 2 * W1);
    c3[k] = pc[k >> 2].c3_3;
  }
  uint32_t ka = k0 + 3 * W0, kb = k1 + 3 * W1;
#pragma unroll
  for (int r = 3; r < 10; ++r) {
    uint64_t p0[8], p1[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      p0[k] = (uint64_t)M0 * c0[k];
      p1[k] = (uint64_t)M1 * c2[k];
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      c0[k] = xor3((uint32_t)(p1[k] >> 32), c1[k], ka);
      c2[k] = xor3((uint32_t)(p0[k] >> 32), c3[k], kb);
      c1[k] = (uint32_t)p1[k];
      c3[k] = (uint32_t)p0[k];
    }
    ka += W0;
    kb += W1;
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) out[k >> 2][k & 3] = Philox4{c0[k], c1[k], c2[k], c3[k]};
}

// ---------------------------------------------------------------------------
// 128 random bits -> the noise of eight elements (paper Sec. 3.4, Eq. 9 and
// Eq. 10), evaluated for all eight at once on nibble planes.  Each element owns
// one nibble position in each of the four words (16 independent bits):
//   |R| = 2 : (b|b) & (8 bits all set)              -> 3/4 * 2^-8
//   |R| = 1 : (b|b) & (b|b) & b, unless |R| = 2     -> (3/4)^2 * 2^-1 * (1 - P(|R|=2))
//   sign    : 1 bit (bit 3 of the x3 nibble; x3 is kept as is)
// Element k of a group owns nibble (k>>1) + 4*(k&1): the two BF16 values of a
// 32-bit register take their bits from the low and the high half of each word.
// ---------------------------------------------------------------------------
struct Noise {
  uint32_t nz;  // bit 0 of each nibble: R != 0
  uint32_t m2;  // bit 0 of each nibble: |R| == 2
  uint32_t x3;  // bit 3 of each nibble: sign
};

__device__ __forceinline__ Noise noise_planes(const Philox4& x) {
  uint32_t all8 = x.x0 & x.x1;
  all8 &= all8 >> 1;
  all8 &= all8 >> 2;                      // bit 0 of each nibble: all 8 bits set
  const uint32_t v = x.x2 | (x.x2 >> 1);  // bit 0: b|b (A), bit 2: b|b (C)
  const uint32_t y = x.x3 | (x.x3 >> 1);  // bit 0: b|b (D)
  Noise n;
  n.m2 = all8 & v & 0x11111111u;
  // (C & D & E) | m2: where m2 is set the element is |R| = 2, elsewhere |R| = 1
  n.nz = ((v >> 2) & y & (x.x3 >> 2) & 0x11111111u) | n.m2;
  n.x3 = x.x3;
  return n;
}

__device__ __forceinline__ Noise group_noise(uint32_t cg, uint32_t row, uint32_t step_lo, uint32_t step_hi,
                                             uint32_t seed_lo, uint32_t seed_hi) {
  return noise_planes(philox4x32_10(cg, row, step_lo, step_hi, seed_lo, seed_hi));
}

// Nibble position of element k of a group.
__host__ __device__ constexpr int element_nibble(int k) { return (k >> 1) + 4 * (k & 1); }

// The packed output format of Sec. 3.4: 4-bit sign-magnitude codes, element k
// in bits 4k..4k+3 (only the noise dump needs it).
__device__ __forceinline__ uint32_t packed_codes(const Noise& n) {
  const uint32_t c = (n.x3 & 0x88888888u) | (n.nz + n.m2);  // per nibble: sign<<3 | |R|
  uint32_t out = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) out |= ((c >> (4 * element_nibble(k))) & 0xFu) << (4 * k);
  return out;
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

// Two fp32 -> packed BF16 pair (lo in bits 0..15), round to nearest even, in
// hardware (v_cvt_pk_bf16_f32; identical to the integer rounding above for
// every finite input).
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
  bf16x2 p = {(__bf16)lo, (__bf16)hi};
  uint32_t u;
  __builtin_memcpy(&u, &p, 4);
  return u;
}

// ---------------------------------------------------------------------------
// Per-block constants of the forward pass.
// ---------------------------------------------------------------------------
struct BlockScale {
  float s32;        // max|w| * 2^(1-b_t), unrounded fp32 (stored; Eq. 4 reuses it)
  uint32_t s_bits;  // bf16_rne(s32) as fp32 bits (sign clear): the step of the PQN
  float x_scale;    // cast: X = 2^(Ea + 1 - EMAX) as fp32
  uint32_t emin_b;  // cast: fp32 exponent field (<<23) of the lowest normal binade of X*format
  uint32_t max_b;   // cast: fp32 bits of max*X (saturation bound)
  bool hw_safe;     // cast: no element of the block can exceed max*X (a + 2s <= max*X)
};

template <int EMAX, int EMIN>
__device__ __forceinline__ void cast_constants(uint32_t a16, BlockScale& b) {
  // Ea = floor(log2 max|w|) from the BF16 exponent field; clamped so that every
  // constant below is a normal fp32 (blocks with max|w| < 2^-100 are outside the
  // supported domain and only have to stay in bounds).
  int ef = (int)(a16 >> 7);
  ef = ef < 27 ? 27 : ef;
  b.x_scale = __uint_as_float((uint32_t)(ef + 1 - EMAX) << 23);
  b.emin_b = (uint32_t)(ef + 1 - EMAX + EMIN) << 23;  // lowest normal = X * 2^EMIN
  b.max_b = ((uint32_t)(ef + 1) << 23) | 0x00600000u; // 1.75 * 2^EMAX * X = 1.75 * 2^(Ea+1)
  const float a = __uint_as_float(a16 << 16);
  b.hw_safe = a + 2.0f * __uint_as_float(b.s_bits) <= __uint_as_float(b.max_b);
}

__device__ __forceinline__ BlockScale block_scale(uint32_t a16, float bt) {
  BlockScale b;
  const float a = __uint_as_float(a16 << 16);
  const float p = exp2_fixed(1.0f - bt);
  b.s32 = a * p;
  b.s_bits = bf16_rne_bits(b.s32) << 16;
  b.x_scale = 1.0f;
  b.emin_b = 0;
  b.max_b = 0;
  b.hw_safe = true;
  return b;
}

// ---------------------------------------------------------------------------
// Block-scaled fp_{e,m} cast (paper Sec. 3.3) of a BF16 value held in fp32, in
// plain arithmetic: round to nearest even onto the grid of spacing
// 2^(max(e_v, emin) - M) by adding and subtracting 2^(23 - M) times that binade
// (the fp32 adder performs the rounding), then saturate and restore the sign.
// ---------------------------------------------------------------------------
template <int M>
__device__ __forceinline__ uint32_t cast_scaled_bits(uint32_t h16, const BlockScale& b) {
  const uint32_t u = h16 << 16;
  const uint32_t au = u & 0x7FFFFFFFu;
  uint32_t eb = au & 0x7F800000u;
  eb = eb > b.emin_b ? eb : b.emin_b;
  const float c = __uint_as_float(eb + ((uint32_t)(23 - M) << 23));
  float r = (__uint_as_float(au) + c) - c;
  r = fminf(r, __uint_as_float(b.max_b));
  return (__float_as_uint(r) | (u & 0x80000000u)) >> 16;
}

// Cast of a packed BF16 pair.  FP8-E4M3 goes through the hardware converters
// (v_cvt_scalef32_pk_fp8_bf16 and back: round to nearest even, gradual
// underflow, division by the power-of-two scale), which produce NaN instead of
// saturating, so they are used only where the block cannot overflow.  FP6-E3M2 is
// cast in arithmetic here; this per-pair form serves the GEMM kernel's operand
// path, while the tile code converts FP6 with the 32-wide hardware converters.
template <int FMT>
__device__ __forceinline__ uint32_t cast_pair(uint32_t pk, const BlockScale& b, bool hw, i16x2& chain) {
  if (FMT == 0) return pk;
  if (FMT == 1 && hw) {
    bf16x2 v;
    __builtin_memcpy(&v, &pk, 4);
    // the converter writes one 16-bit half of its destination and keeps the other:
    // chaining the previous result as "old" avoids a register clear per call
    chain = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(chain, v, b.x_scale, false);
    uint32_t cu;
    __builtin_memcpy(&cu, &chain, 4);
    const bf16x2 r = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(cu, b.x_scale, false);
    uint32_t ru;
    __builtin_memcpy(&ru, &r, 4);
    return ru;
  }
  constexpr int M = (FMT == 1) ? 3 : 2;
  return cast_scaled_bits<M>(pk & 0xFFFFu, b) | (cast_scaled_bits<M>(pk >> 16, b) << 16);
}

// Byte i of x as fp32 (v_cvt_f32_ubyte<i>).  The empty asm hides what is known
// about the other bits of x, so the byte extraction is not rewritten into a
// shift-and-mask pair.
__device__ __forceinline__ uint32_t opaque(uint32_t x) {
  asm volatile("" : "+v"(x));
  return x;
}
template <int I>
__device__ __forceinline__ float byte_to_f32(uint32_t x) {
  return (float)((x >> (8 * I)) & 0xFFu);
}

// ---------------------------------------------------------------------------
// Eq. 3 + cast on one 16-byte group (8 BF16 in 4 registers).  PQN = R * s is
// formed in sign-magnitude: |R| * s is exact and the sign bit is placed as is
// (R = -0 gives -0.0); the fp32 fused multiply-add followed by one RNE to BF16
// equals the exact BF16 sum.
// ---------------------------------------------------------------------------
struct GroupMagnitudes {
  float m[8];  // |R| of element k as fp32
};

__device__ __forceinline__ GroupMagnitudes group_magnitudes(const Noise& n) {
  const uint32_t mag = n.nz + n.m2;  // per nibble: |R| in {0, 1, 2}
  const uint32_t me = opaque(mag & 0x0F0F0F0Fu);         // byte i: |R| of nibble 2i
  const uint32_t mo = opaque((mag >> 4) & 0x0F0F0F0Fu);  // byte i: |R| of nibble 2i+1
  // element 2d sits in nibble d, element 2d+1 in nibble d+4
  return GroupMagnitudes{{byte_to_f32<0>(me), byte_to_f32<2>(me), byte_to_f32<0>(mo), byte_to_f32<2>(mo),
                          byte_to_f32<1>(me), byte_to_f32<3>(me), byte_to_f32<1>(mo), byte_to_f32<3>(mo)}};
}

// bf16_rne(w + R * s) for elements 2d and 2d+1 of a group (register d), packed.
template <int D>
__device__ __forceinline__ uint32_t sampled_pair(uint32_t wd, const GroupMagnitudes& g, const Noise& n,
                                                 const BlockScale& b) {
  constexpr int n_lo = D, n_hi = D + 4;
  // s with the sign bit of the nibble: (x3 << sh) & 0x80000000 | s, one shift and one bit-op
  const uint32_t sh_lo = n.x3 << (28 - 4 * n_lo);
  const uint32_t sh_hi = (n_hi == 7) ? n.x3 : (n.x3 << (28 - 4 * n_hi));
  const float s_lo = __uint_as_float(__builtin_amdgcn_bitop3_b32(sh_lo, 0x80000000u, b.s_bits, 0xEA));
  const float s_hi = __uint_as_float(__builtin_amdgcn_bitop3_b32(sh_hi, 0x80000000u, b.s_bits, 0xEA));
  const float w_lo = __uint_as_float(wd << 16), w_hi = __uint_as_float(wd & 0xFFFF0000u);
  const float sum_lo = __fmaf_rn(g.m[2 * D], s_lo, w_lo);
  const float sum_hi = __fmaf_rn(g.m[2 * D + 1], s_hi, w_hi);
  return pack_bf16_rne(sum_lo, sum_hi);
}

template <int FMT>
__device__ __forceinline__ u32x4 sample_group(const u32x4 w, const Noise& n, const BlockScale& b, bool hw) {
  const GroupMagnitudes g = group_magnitudes(n);
  i16x2 chain = {0, 0};
  u32x4 out;
  out[0] = cast_pair<FMT>(sampled_pair<0>(w[0], g, n, b), b, hw, chain);
  out[1] = cast_pair<FMT>(sampled_pair<1>(w[1], g, n, b), b, hw, chain);
  out[2] = cast_pair<FMT>(sampled_pair<2>(w[2], g, n, b), b, hw, chain);
  out[3] = cast_pair<FMT>(sampled_pair<3>(w[3], g, n, b), b, hw, chain);
  return out;
}

// ---------------------------------------------------------------------------
// The same group as microscaling element codes (OCP MX: FP8 E4M3 with bias 7,
// FP6 E3M2 with bias 3) of q / X, X the block's power-of-two scale.
// ---------------------------------------------------------------------------
struct MxCodes {
  uint32_t lo, hi;  // FP8: 8 code bytes.  FP6: 8 codes of 6 bits, element k in bits [6k, 6k+6) of hi:lo
};

// Code of a BF16 value under the block scale, in plain arithmetic.  Adding
// 2^(23 - M) times the binade (the binade of the value, or the lowest normal one
// of X * format below it) makes the fp32 adder round the value to nearest even
// onto the format's grid and leaves the count of grid steps, k, in the low
// mantissa bits; the code is that count on top of the binade's first code.
template <int M, int EBITS, uint32_t MAXCODE>
__device__ __forceinline__ uint32_t encode_scaled(uint32_t h16, const BlockScale& b) {
  const uint32_t u = h16 << 16;
  const uint32_t au = u & 0x7FFFFFFFu;
  uint32_t eb = au & 0x7F800000u;
  eb = eb > b.emin_b ? eb : b.emin_b;
  const uint32_t cb = eb + ((uint32_t)(23 - M) << 23);
  const float t = __uint_as_float(au) + __uint_as_float(cb);
  const uint32_t k = __float_as_uint(t) - cb;            // 0 .. 2^(M+1)
  uint32_t code = ((eb - b.emin_b) >> (23 - M)) + k;     // (E - 1) << M, plus k
  code = code < MAXCODE ? code : MAXCODE;                // saturate at the largest finite code
  return code | ((u >> 31) << (M + EBITS));
}

// FP8-E4M3 codes of one group.  (FP6-E3M2 codes come from the 32-wide converter, a lane's
// whole tile at a time: see fwd_tile.)
__device__ __forceinline__ MxCodes sample_group_mx_fp8(const u32x4 w, const Noise& n, const BlockScale& b, bool hw) {
  const GroupMagnitudes g = group_magnitudes(n);
  const uint32_t pk[4] = {sampled_pair<0>(w[0], g, n, b), sampled_pair<1>(w[1], g, n, b),
                          sampled_pair<2>(w[2], g, n, b), sampled_pair<3>(w[3], g, n, b)};
  MxCodes c;
  if (hw) {
    // hardware converter: rounds to nearest even under the scale; each call fills one
    // 16-bit half of its destination register
    bf16x2 v[4];
    __builtin_memcpy(v, pk, 16);
    i16x2 a = {0, 0}, h = {0, 0};
    a = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(a, v[0], b.x_scale, false);
    a = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(a, v[1], b.x_scale, true);
    h = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(h, v[2], b.x_scale, false);
    h = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(h, v[3], b.x_scale, true);
    __builtin_memcpy(&c.lo, &a, 4);
    __builtin_memcpy(&c.hi, &h, 4);
    return c;
  }
  // the block can exceed 448 X, where the converter would give NaN: saturating arithmetic form
  uint32_t e[8];
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    e[2 * d] = encode_scaled<3, 4, 0x7Eu>(pk[d] & 0xFFFFu, b);
    e[2 * d + 1] = encode_scaled<3, 4, 0x7Eu>(pk[d] >> 16, b);
  }
  c.lo = e[0] | (e[1] << 8) | (e[2] << 16) | (e[3] << 24);
  c.hi = e[4] | (e[5] << 8) | (e[6] << 16) | (e[7] << 24);
  return c;
}

// ---------------------------------------------------------------------------
// Comparison noise bases (paper Sec. 4): the same pipeline with R drawn as a BF16
// U(-0.5, 0.5) value (the paper's "DiffQ" extension) or as the exact rounded normal
// round(N(0,1) / 2) from a Box-Muller transform (the "bm" baseline of its forward
// unit benchmark).  Both take the group's Philox call as it is; only the map from
// the 128 bits to the eight R differs.
//   uniform:    element k owns byte k % 4 of word k / 4; R = (2 byte - 255) / 512, one of the
//               256 midpoints of a 1/256 grid on (-0.5, 0.5), each a BF16 value.  R * s is not
//               exact here and is rounded to BF16 before the add (the BF16 operator of Sec. 3.3).
//   Box-Muller: the pair of elements (2d, 2d + 1) owns word d; u1 = (low half + 0.5) / 2^16,
//               u2 = (high half + 0.5) / 2^16, z = sqrt(-2 ln u1) (cos, sin)(2 pi u2),
//               R = rint(z / 2).  Floating point decides an integer here, so the fp32 operations
//               and their order are fixed (no contraction, correctly rounded square root).
// ---------------------------------------------------------------------------
constexpr int kBasisBits = 0, kBasisUniform = 1, kBasisBoxMuller = 2;

// R of elements 2d and 2d + 1 of a group as fp32 (exact), uniform basis.
template <int D>
__device__ __forceinline__ void uniform_pair(const Philox4& x, float& r_lo, float& r_hi) {
  const uint32_t word = (D >> 1) ? x.x1 : x.x0;   // elements 0..3 in x0, 4..7 in x1
  const float step = __uint_as_float(0x3B800000u), off = __uint_as_float(0xBEFF0000u);   // 2^-8, -255/512
  r_lo = __fmaf_rn(byte_to_f32<2 * (D & 1)>(word), step, off);
  r_hi = __fmaf_rn(byte_to_f32<2 * (D & 1) + 1>(word), step, off);
}

// ln(u) for u = (k + 0.5) / 2^16: u = m 2^e with m in [1/sqrt2, sqrt2), ln u = e ln2 + f P(f), f = m - 1,
// P of degree 8 evaluated by Horner's rule with fused multiply-adds.
__device__ __forceinline__ float bm_log(float u) {
  const uint32_t ub = __float_as_uint(u);
  int e = (int)(ub >> 23) - 127;
  float m = __uint_as_float((ub & 0x007FFFFFu) | 0x3F800000u);
  if (m > __uint_as_float(0x3FB504F3u)) {
    m = __fmul_rn(m, 0.5f);
    e += 1;
  }
  const float f = __fsub_rn(m, 1.0f);
  float p = __uint_as_float(0x3DB31375u);
  p = __fmaf_rn(p, f, __uint_as_float(0xBE13394Fu));
  p = __fmaf_rn(p, f, __uint_as_float(0x3E191428u));
  p = __fmaf_rn(p, f, __uint_as_float(0xBE2994DFu));
  p = __fmaf_rn(p, f, __uint_as_float(0x3E4C5C05u));
  p = __fmaf_rn(p, f, __uint_as_float(0xBE8002D3u));
  p = __fmaf_rn(p, f, __uint_as_float(0x3EAAABC8u));
  p = __fmaf_rn(p, f, __uint_as_float(0xBEFFFFFCu));
  p = __fmaf_rn(p, f, 1.0f);
  return __fmaf_rn((float)e, __uint_as_float(0x3F317218u), __fmul_rn(p, f));
}

// R of the two elements that own `word`, as fp32 in {-2, -1, -0, 0, 1, 2}.
__device__ __forceinline__ void box_muller_pair(uint32_t word, float& r_lo, float& r_hi) {
  const float u1 = __fmul_rn(__fadd_rn((float)(word & 0xFFFFu), 0.5f), __uint_as_float(0x37800000u));
  const float L = __fmul_rn(-2.0f, bm_log(u1));
  const float r = __builtin_sqrtf(L);   // correctly rounded
  const uint32_t hi = word >> 16, q = hi >> 14, j = hi & 0x3FFFu;
  // angle = q pi/2 + pi/4 + t, t = (2 j + 1 - 16384) fl(pi / 65536) in (-pi/4, pi/4)
  const float t = __fmul_rn((float)(2 * (int)j + 1 - 16384), __uint_as_float(0x38490FDBu));
  const float t2 = __fmul_rn(t, t);
  float sp = __uint_as_float(0xB94D6501u);
  sp = __fmaf_rn(sp, t2, __uint_as_float(0x3C088615u));
  sp = __fmaf_rn(sp, t2, __uint_as_float(0xBE2AAAA9u));
  const float st = __fmaf_rn(__fmul_rn(t, t2), sp, t);
  float cp = __uint_as_float(0x37CD3809u);
  cp = __fmaf_rn(cp, t2, __uint_as_float(0xBAB60706u));
  cp = __fmaf_rn(cp, t2, __uint_as_float(0x3D2AAAA6u));
  cp = __fmaf_rn(cp, t2, __uint_as_float(0xBF000000u));
  const float ct = __fmaf_rn(t2, cp, 1.0f);
  const float h = __uint_as_float(0x3F3504F3u);
  const float c = __fmul_rn(__fsub_rn(ct, st), h), sn = __fmul_rn(__fadd_rn(ct, st), h);
  // q quarter turns: (c, s) -> (-s, c) -> (-c, -s) -> (s, -c); negation is a sign-bit flip
  const uint32_t cb = __float_as_uint(c), sb = __float_as_uint(sn);
  const uint32_t cq = ((q & 1) ? sb : cb) ^ (((q + 1) & 2) << 30);
  const uint32_t sq = ((q & 1) ? cb : sb) ^ ((q & 2) << 30);
  r_lo = __builtin_rintf(__fmul_rn(0.5f, __fmul_rn(r, __uint_as_float(cq))));
  r_hi = __builtin_rintf(__fmul_rn(0.5f, __fmul_rn(r, __uint_as_float(sq))));
}

// R of elements 2d, 2d + 1 under a comparison basis.
template <int BASIS, int D>
__device__ __forceinline__ void basis_pair(const Philox4& x, float& r_lo, float& r_hi) {
  if (BASIS == kBasisUniform) {
    uniform_pair<D>(x, r_lo, r_hi);
  } else {
    box_muller_pair(D == 0 ? x.x0 : D == 1 ? x.x1 : D == 2 ? x.x2 : x.x3, r_lo, r_hi);
  }
}

// bf16_rne(w + PQN) for elements 2d, 2d + 1 under a comparison basis: PQN = bf16_rne(R * s) (exact for the
// integer R of the Box-Muller basis, where the fused multiply-add gives the same bits in one step).
template <int BASIS, int D>
__device__ __forceinline__ uint32_t sampled_pair_basis(uint32_t wd, const Philox4& x, const BlockScale& b) {
  float r_lo, r_hi;
  basis_pair<BASIS, D>(x, r_lo, r_hi);
  const float s = __uint_as_float(b.s_bits);
  const float w_lo = __uint_as_float(wd << 16), w_hi = __uint_as_float(wd & 0xFFFF0000u);
  if (BASIS == kBasisUniform) {
    const uint32_t pq = pack_bf16_rne(__fmul_rn(r_lo, s), __fmul_rn(r_hi, s));
    return pack_bf16_rne(__fadd_rn(w_lo, __uint_as_float(pq << 16)), __fadd_rn(w_hi, __uint_as_float(pq & 0xFFFF0000u)));
  }
  return pack_bf16_rne(__fmaf_rn(r_lo, s, w_lo), __fmaf_rn(r_hi, s, w_hi));
}

// The eight R of a group under a comparison basis as four packed BF16 pairs (every R is a BF16 value).
template <int BASIS>
__device__ __forceinline__ u32x4 basis_group_bf16(const Philox4& x) {
  float lo[4], hi[4];
  basis_pair<BASIS, 0>(x, lo[0], hi[0]);
  basis_pair<BASIS, 1>(x, lo[1], hi[1]);
  basis_pair<BASIS, 2>(x, lo[2], hi[2]);
  basis_pair<BASIS, 3>(x, lo[3], hi[3]);
  return u32x4{pack_bf16_rne(lo[0], hi[0]), pack_bf16_rne(lo[1], hi[1]), pack_bf16_rne(lo[2], hi[2]), pack_bf16_rne(lo[3], hi[3])};
}

// sum over one group of g .* R under a comparison basis (products exact, fp32 accumulation, fixed order).
template <int BASIS>
__device__ __forceinline__ float dot_group_basis(const u32x4 g, const Philox4& x, float acc) {
  const u32x4 r = basis_group_bf16<BASIS>(x);
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t gd = g[d], rd = r[d];
    bf16x2 gv, rv;
    __builtin_memcpy(&gv, &gd, 4);
    __builtin_memcpy(&rv, &rd, 4);
    acc = __builtin_amdgcn_fdot2_f32_bf16(gv, rv, acc, false);
  }
  return acc;
}

// sum over one group of g .* (2R), two elements per v_dot2 (products exact, fp32
// accumulation).  2R in {0, +-2, +-4} has the BF16 patterns sign<<15 | nz<<14 |
// m2<<7.  The three bits of every element are first moved to the top of a byte
// (bits 7, 6 of a "high" byte: sign, nz; bit 7 of a "low" byte: m2), separately for
// the elements in even and in odd nibbles; one byte permute then assembles the
// pattern pair of register d from the bytes of nibbles d and d + 4.
__device__ __forceinline__ float dot_group_2r(const u32x4 g, const Noise& n, float acc) {
  const uint32_t a = (n.x3 & 0x88888888u) | (n.nz << 2);   // per nibble: bit 3 sign, bit 2 nz
  const uint32_t hi_odd = a & 0xC0C0C0C0u;                  // byte i: element of nibble 2i + 1
  const uint32_t hi_even = (a << 4) & 0xC0C0C0C0u;          // byte i: element of nibble 2i
  const uint32_t lo_odd = (n.m2 << 3) & 0x80808080u;
  const uint32_t lo_even = (n.m2 << 7) & 0x80808080u;
  // v_perm_b32 selectors: result bytes (lo, hi, lo, hi) from byte j and j + 2 of the two words
  const uint32_t pat[4] = {__builtin_amdgcn_perm(hi_even, lo_even, 0x06020400u),   // nibbles 0, 4
                           __builtin_amdgcn_perm(hi_odd, lo_odd, 0x06020400u),     // nibbles 1, 5
                           __builtin_amdgcn_perm(hi_even, lo_even, 0x07030501u),   // nibbles 2, 6
                           __builtin_amdgcn_perm(hi_odd, lo_odd, 0x07030501u)};    // nibbles 3, 7
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t gd = g[d];
    bf16x2 gv, rv;
    __builtin_memcpy(&gv, &gd, 4);
    __builtin_memcpy(&rv, &pat[d], 4);
    acc = __builtin_amdgcn_fdot2_f32_bf16(gv, rv, acc, false);
  }
  return acc;
}

// ---------------------------------------------------------------------------
// Cross-lane reductions over the 32 lanes of a wavefront that share a 32x32
// block.  Lane = 8 * row_in_8 + column_group; a block owns column groups
// {0..3} or {4..7}, so its lanes differ in lane bits 0, 1, 3, 4, 5.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

__device__ __forceinline__ uint32_t block_max_u32(uint32_t v) {
  v = max(v, dpp_u32<0xB1>(v));   // quad_perm [1,0,3,2]: lane ^ 1
  v = max(v, dpp_u32<0x4E>(v));   // quad_perm [2,3,0,1]: lane ^ 2
  v = max(v, dpp_u32<0x128>(v));  // row_ror 8: lane ^ 8 within a row of 16
  v = max(v, (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F));  // lane ^ 16
  v = max(v, (uint32_t)__shfl_xor((int)v, 32));
  return v;
}

__device__ __forceinline__ float block_sum_f32(float v) {
  v += __uint_as_float(dpp_u32<0xB1>(__float_as_uint(v)));
  v += __uint_as_float(dpp_u32<0x4E>(__float_as_uint(v)));
  v += __uint_as_float(dpp_u32<0x128>(__float_as_uint(v)));
  v += __uint_as_float((uint32_t)__builtin_amdgcn_ds_swizzle((int)__float_as_uint(v), 0x401F));
  v += __shfl_xor(v, 32);
  return v;
}

// max|w| of a 16-byte group, as BF16 magnitude bits in both halves of a register.
__device__ __forceinline__ uint32_t absmax_pk(const u32x4 w, uint32_t m) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t a = w[d] & 0x7FFF7FFFu;
    u16x2 x, y;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &m, 4);
    const u16x2 z = __builtin_elementwise_max(x, y);
    __builtin_memcpy(&m, &z, 4);
  }
  return m;
}

}  // namespace gws
