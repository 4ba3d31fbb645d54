/*
 * GaussWS CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of the Gaussian weight
 * sampling forward/backward (paper Sec. 3.2 Eq. 3 and Eq. 4, noise basis of
 * Sec. 3.4 Eq. 10, FP cast fp_{e,m} of Sec. 3.3) used to check the HIP
 * kernels.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it; the product path never does.  It shares no code, header or
 * table with the HIP path: every constant below is typed in here on its own.
 *
 * Every function follows the steps in the paper's order, one element at a
 * time, with no blocking or fusion beyond the 32x32 block the method itself
 * defines.  Floating point that decides a stored bit pattern (block scale,
 * BF16 add, casts) is emulated on integers or evaluated with explicitly
 * sequenced fp32 operations so the result is a single defined bit pattern;
 * reductions (Eq. 4's block sum, the GEMM) are done in fp64.
 *
 * Parity pins (tests/test_oracle_*.py): Philox known-answer vectors, the
 * exhaustive 2^16 enumeration of the bit->R map against Eq. 10's closed form,
 * torch CPU bfloat16 adds, torch CPU float8_e4m3fn casts, brute-force nearest
 * search over the enumerated FP6-E3M2 / FP8-E4M3 code sets, hand-worked
 * blocks, Table C.1, finite differences of Eq. 3 for Eq. 4, the end points
 * of Eq. 11 and finite differences of Eq. 12; for the MX output torch's
 * float8 byte patterns, the element-format figures of the OCP Microscaling
 * specification, numpy's bit unpacking and the BF16-container output itself;
 * for the comparison bases the exact moments of the enumerated uniform values,
 * torch CPU bfloat16 products, the fp64 Box-Muller formula, and the cell
 * probabilities of the rounded normal from erf.
 * Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define GWSO_BL 32 /* b_l: square block edge, Sec. 3.2 */

enum { GWSO_FMT_BF16 = 0, GWSO_FMT_FP8_E4M3 = 1, GWSO_FMT_FP6_E3M2 = 2 };

/* ------------------------------------------------------------------ */
/* Threads (only used by the benchmark's cpu_baseline leg)             */
/* ------------------------------------------------------------------ */
int gwso_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
  return omp_get_max_threads();
#else
  (void)n;
  return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Philox4x32 (Salmon et al., SC'11), the counter-based bit source the  */
/* paper names in Sec. 3.4.  `rounds` = 10 is the standard generator.   */
/* ------------------------------------------------------------------ */
void gwso_philox4x32(const uint32_t ctr[4], const uint32_t key[2], int rounds,
                     uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < rounds; ++r) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Per-tensor seed: replaces the paper's stateful per-layer PRNG (Sec. 3.6,
 * "Managing seed") by a pure function of (user seed, tensor id).            */
uint64_t gwso_derive_seed(uint64_t user_seed, uint64_t tensor_id) {
  uint32_t ctr[4] = {(uint32_t)tensor_id, (uint32_t)(tensor_id >> 32), 0x47575331u, 0u};
  uint32_t key[2] = {(uint32_t)user_seed, (uint32_t)(user_seed >> 32)};
  uint32_t o[4];
  gwso_philox4x32(ctr, key, 10, o);
  return (uint64_t)o[0] | ((uint64_t)o[1] << 32);
}

/* ------------------------------------------------------------------ */
/* Random bits -> R (Sec. 3.4, Eq. 9 and Eq. 10).                      */
/* An element owns 16 independent bits, given here as four nibbles      */
/* n0..n3.  Built only from AND/OR of independent bits:                 */
/*   |R|=2  <=> (b or b) and (8 bits all set)          : 3/4 * 2^-8     */
/*   |R|=1  <=> (b or b) and (b or b) and b, not |R|=2 : (3/4)^2 * 2^-1 */
/*   sign   <=> one bit                                                 */
/* Returns the 4-bit sign-magnitude code (sign<<3 | magnitude).         */
/* ------------------------------------------------------------------ */
int gwso_nibbles_to_code(unsigned n0, unsigned n1, unsigned n2, unsigned n3) {
  int all8 = (n0 == 0xFu) && (n1 == 0xFu);
  int A = (n2 & 0x3u) != 0;
  int C = (n2 & 0xCu) != 0;
  int D = (n3 & 0x3u) != 0;
  int E = (n3 >> 2) & 1;
  int S = (n3 >> 3) & 1;
  int mag2 = all8 && A;
  int mag1 = C && D && E && !mag2;
  return (S << 3) | (mag2 << 1) | mag1;
}

/* code -> integer R in {-2,-1,0,1,2} */
int gwso_code_to_r(int code) {
  int mag = code & 3;
  return (code & 8) ? -mag : mag;
}

/* The four Philox words of the group of 8 row-contiguous elements that
 * holds element (i, j): counter = (column group j>>3, row i, step lo, step hi),
 * key = per-tensor seed.  Forward and backward call this with the same
 * (seed, step), which is what makes R identical in both (Sec. 3.5, 3.6).     */
static void group_words(int64_t i, int64_t cg, uint64_t seed, uint64_t step,
                        uint32_t x[4]) {
  uint32_t ctr[4] = {(uint32_t)cg, (uint32_t)i, (uint32_t)step, (uint32_t)(step >> 32)};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  gwso_philox4x32(ctr, key, 10, x);
}

/* Which nibble of each Philox word belongs to element k (= j & 7) of a group.
 * Sec. 3.4 fixes 4 bits per element and 8 elements per 32-bit word but not which
 * bits go to which element, so the assignment is a free choice; it is frozen as:
 * each 32-bit word is seen as two 16-bit halves, the low half serving the even
 * elements and the high half the odd ones; pair k>>1 takes nibble k>>1 of its half. */
int gwso_element_nibble(int k) { return (k >> 1) + 4 * (k & 1); }

static int element_code(const uint32_t x[4], int k) {
  int sh = 4 * gwso_element_nibble(k);
  return gwso_nibbles_to_code((x[0] >> sh) & 0xFu, (x[1] >> sh) & 0xFu,
                              (x[2] >> sh) & 0xFu, (x[3] >> sh) & 0xFu);
}

/* Noise of a whole [rows x cols] tensor.
 *   r      : int8 [rows x cols] (may be NULL), R values
 *   packed : u32  [rows x ceil(cols/8)] (may be NULL), 8 codes per word,
 *            element k of the group in bits 4k..4k+3 (Sec. 3.4, packed format)
 * (row0, col0): where this tensor sits inside a larger one (col0 a multiple of
 * 8); they only shift the counter, so a shard sees the full tensor's noise.     */
void gwso_noise(int64_t rows, int64_t cols, int64_t row0, int64_t col0, uint64_t seed,
                uint64_t step, int8_t* r, uint32_t* packed) {
  int64_t ngrp = (cols + 7) / 8;
  for (int64_t i = 0; i < rows; ++i) {
    for (int64_t cg = 0; cg < ngrp; ++cg) {
      uint32_t x[4];
      group_words(row0 + i, col0 / 8 + cg, seed, step, x);
      uint32_t word = 0;
      for (int k = 0; k < 8; ++k) {
        int code = element_code(x, k);
        word |= (uint32_t)code << (4 * k);
        int64_t j = cg * 8 + k;
        if (r && j < cols) r[i * cols + j] = (int8_t)gwso_code_to_r(code);
      }
      if (packed) packed[i * ngrp + cg] = word;
    }
  }
}

/* ------------------------------------------------------------------ */
/* BF16 helpers: values travel as uint16 bit patterns.                  */
/* ------------------------------------------------------------------ */
static float bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

static uint32_t f32_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  return u;
}

/* fp32 -> BF16, round to nearest, ties to even (finite inputs). */
uint16_t gwso_bf16_rne(float f) {
  uint32_t u = f32_bits(f);
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  return (uint16_t)(u >> 16);
}

/* Exact BF16 + BF16 -> BF16 with ONE round-to-nearest-even, on integers.
 * Operands are decoded to sign / exponent / 8-bit significand; the smaller
 * one is aligned with a sticky bit; the exact sum is normalised and rounded
 * once.  Finite inputs; overflow gives infinity.  Sign of an exact zero sum
 * follows IEEE 754 (x + (-x) = +0; (-0) + (-0) = -0).                        */
uint16_t gwso_bf16_add(uint16_t a, uint16_t b) {
  int sa = a >> 15, sb = b >> 15;
  int ea = (a >> 7) & 0xFF, eb = (b >> 7) & 0xFF;
  uint64_t ma = a & 0x7Fu, mb = b & 0x7Fu;
  if (ea) ma |= 0x80u; else ea = 1; /* subnormal: exponent of the lowest binade */
  if (eb) mb |= 0x80u; else eb = 1;
  /* order so that |a| >= |b| */
  if (eb > ea || (eb == ea && mb > ma)) {
    int t = sa; sa = sb; sb = t;
    t = ea; ea = eb; eb = t;
    uint64_t m = ma; ma = mb; mb = m;
  }
  if (ma == 0) { /* both zero */
    return (uint16_t)((sa && sb) ? 0x8000u : 0x0000u);
  }
  /* fixed point with 40 fraction bits below the BF16 lsb of a */
  const int G = 40;
  uint64_t A = ma << G, B;
  int sh = ea - eb;
  int sticky = 0;
  if (sh >= G + 8) { B = 0; sticky = (mb != 0); }
  else {
    B = mb << G;
    if (sh > 0) {
      sticky = (B & ((1ull << sh) - 1)) != 0; /* always 0 for sh <= G */
      B >>= sh;
    }
  }
  uint64_t S;
  if (sa == sb) S = A + B;
  else {
    S = A - B;
    if (sticky) { S -= 1; } /* borrow: true value lies strictly between S-1 and S */
  }
  if (S == 0 && !sticky) return 0x0000u; /* exact cancellation -> +0 (RNE mode) */
  /* S (plus sticky) * 2^(ea - 127 - 7 - G) is the exact magnitude */
  int e = ea; /* exponent field if the leading one sits at bit G+7 */
  while (S >= (1ull << (G + 8))) { sticky |= (int)(S & 1); S >>= 1; e += 1; }
  while (S < (1ull << (G + 7)) && e > 1) { S <<= 1; e -= 1; }
  /* round to 8 significant bits (or fewer when subnormal: e == 1, no hidden bit) */
  uint64_t keep = S >> G;
  uint64_t rem = S & ((1ull << G) - 1);
  uint64_t half = 1ull << (G - 1);
  int up = (rem > half) || (rem == half && (sticky || (keep & 1)));
  keep += (uint64_t)up;
  if (keep >= 0x100u) { keep >>= 1; e += 1; }       /* carried into the next binade */
  uint32_t field;
  if (keep < 0x80u) field = (uint32_t)keep;          /* subnormal or zero */
  else field = ((uint32_t)e << 7) | (uint32_t)(keep & 0x7Fu);
  if (keep >= 0x80u && e >= 0xFF) field = 0x7F80u;   /* overflow -> inf */
  return (uint16_t)(((uint32_t)sa << 15) | field);
}

/* ------------------------------------------------------------------ */
/* 2^t for the block scale 2^(1 - b_t) of Eq. 3, as ONE defined fp32    */
/* function (b_t is a real-valued trained parameter, Sec. 3.6):         */
/*   n = rint(t), f = t - n in [-1/2, 1/2] (exact),                     */
/*   p = degree-6 Horner polynomial in f with fused multiply-adds,      */
/*   result = p * 2^n.                                                  */
/* Exact for integer t; below 1 ulp from the true 2^t elsewhere.        */
/* ------------------------------------------------------------------ */
float gwso_exp2(float t) {
  static const uint32_t cbits[7] = {0x3F800000u, 0x3F317218u, 0x3E75FDF0u, 0x3D6357B6u,
                                    0x3C1D950Eu, 0x3AAF844Bu, 0x39222002u};
  float c[7];
  memcpy(c, cbits, sizeof c);
  float n = rintf(t);            /* ties to even (default rounding mode) */
  float f = t - n;
  float p = c[6];
  for (int i = 5; i >= 0; --i) p = fmaf(p, f, c[i]);
  return ldexpf(p, (int)n);
}

/* ------------------------------------------------------------------ */
/* fp_{e,m} cast of Sec. 3.3, read as a block-scaled (MX-style) cast:   */
/* the format's top binade is placed one above the binade of max|w|,    */
/* the headroom binade that w_hat can reach (proof of Prop. 3).         */
/*   X = 2^(Ea + 1 - emax),  q = X * sat( rne_{e,m}( v / X ) )          */
/* with gradual underflow, ties to even, sign of zero kept, saturation   */
/* to +-max*X.  v and q are BF16 bit patterns; q is exactly BF16-        */
/* representable.  Ea = floor(log2 max|w|) of the block.                 */
/* ------------------------------------------------------------------ */
static void fmt_params(int fmt, int* emax, int* emin, int* m, double* maxv) {
  if (fmt == GWSO_FMT_FP8_E4M3) { *emax = 8; *emin = -6; *m = 3; *maxv = 448.0; }
  else { *emax = 4; *emin = -2; *m = 2; *maxv = 28.0; } /* FP6_E3M2 */
}

uint16_t gwso_cast(uint16_t v16, int Ea, int fmt) {
  if (fmt == GWSO_FMT_BF16) return v16;
  int emax, emin, m;
  double maxv;
  fmt_params(fmt, &emax, &emin, &m, &maxv);
  int xe = Ea + 1 - emax;
  double v = (double)bf16_to_f32(v16);
  double y = ldexp(v, -xe);              /* exact: power-of-two scaling in fp64 */
  double ay = fabs(y);
  double q = 0.0;
  if (ay != 0.0) {
    int e = ilogb(ay);
    if (e < emin) e = emin;              /* subnormal range of the target */
    double quantum = ldexp(1.0, e - m);
    q = quantum * nearbyint(ay / quantum); /* RNE; both steps exact */
    if (q > maxv) q = maxv;              /* saturate */
  }
  double out = ldexp(q, xe);
  float of = (float)out;                 /* exact */
  uint16_t r = (uint16_t)(f32_bits(of) >> 16);
  return (uint16_t)((v16 & 0x8000u) | (r & 0x7FFFu));
}

/* Array forms of the two scalar routines above, so that a test can sweep all
 * 65 536 BF16 patterns without a Python-level loop. */
void gwso_bf16_add_n(const uint16_t* a, const uint16_t* b, uint16_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = gwso_bf16_add(a[i], b[i]);
}

void gwso_cast_n(const uint16_t* v, int Ea, int fmt, uint16_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = gwso_cast(v[i], Ea, fmt);
}

void gwso_exp2_n(const float* t, float* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = gwso_exp2(t[i]);
}

/* floor(log2 a) for a positive finite BF16 value (subnormals included). */
static int floor_log2_bf16(uint16_t a16) {
  return ilogb((double)bf16_to_f32(a16));
}

/* ------------------------------------------------------------------ */
/* Alternative noise bases: the systems the paper compares GaussWS with */
/* (Sec. 4: "DiffQ" = the same pipeline with a BF16 U(-0.5, 0.5) basis;  */
/* Sec. 4 "Overhead": "bm" = the exact rounded normal round(N(0,1)/2)    */
/* from a Box-Muller transform).  The paper does not say how either is   */
/* drawn from the random integers; the readings taken here:              */
/*  - both use the same Philox call per group of 8 elements as the bit   */
/*    basis (same counter, same key), so only the map bits -> R differs;  */
/*  - uniform: element k of the group takes byte (k & 3) of word k >> 2   */
/*    and R = (2 * byte - 255) / 512: the 256 midpoints of a 1/256 grid   */
/*    on (-0.5, 0.5), each exactly a BF16 value, mean exactly 0;          */
/*  - Box-Muller: the pair of elements (2d, 2d+1) takes word d,           */
/*    u1 = (low half + 0.5) / 2^16, u2 = (high half + 0.5) / 2^16,        */
/*    z = sqrt(-2 ln u1) * (cos, sin)(2 pi u2), R = rint(z / 2) (ties to   */
/*    even), all in fp32 as ONE defined sequence of operations (below),    */
/*    because here floating point decides an integer.                      */
/* With the uniform basis R * s is not exact, and the BF16 operator of    */
/* Sec. 3.3 rounds it: PQN = bf16(R * s), w_hat = bf16(w + PQN).           */
/* ------------------------------------------------------------------ */
enum { GWSO_BASIS_BITS = 0, GWSO_BASIS_UNIFORM = 1, GWSO_BASIS_BOX_MULLER = 2 };

static float f32_from_bits(uint32_t u) {
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* (2 * byte - 255) / 512 as a BF16 bit pattern (exact: an odd numerator below 256 has 8 significant bits). */
uint16_t gwso_uniform_bf16(unsigned byte) {
  float v = ((float)(2 * (int)(byte & 0xFFu) - 255)) / 512.0f; /* exact */
  return (uint16_t)(f32_bits(v) >> 16);
}

/* BF16 * BF16 -> BF16, one round-to-nearest-even: the fp32 product of two 8-bit significands is exact. */
uint16_t gwso_bf16_mul(uint16_t a, uint16_t b) {
  return gwso_bf16_rne(bf16_to_f32(a) * bf16_to_f32(b));
}

/* ln(u) for u = (k + 0.5) / 2^16, k = 0 .. 65535, in fp32: u = m * 2^e with m in [1/sqrt2, sqrt2),
 * ln u = e * ln2 + f * P(f), f = m - 1, P a degree-8 polynomial (Horner, fused multiply-adds).
 * Within 2e-8 + 1 ulp of the true logarithm. */
static float bm_log(float u) {
  static const uint32_t cb[9] = {0x3F800000u, 0xBEFFFFFCu, 0x3EAAABC8u, 0xBE8002D3u, 0x3E4C5C05u,
                                 0xBE2994DFu, 0x3E191428u, 0xBE13394Fu, 0x3DB31375u};
  uint32_t ub = f32_bits(u);
  int e = (int)(ub >> 23) - 127;
  float m = f32_from_bits((ub & 0x007FFFFFu) | 0x3F800000u);   /* [1, 2) */
  if (m > f32_from_bits(0x3FB504F3u)) { m = m * 0.5f; e += 1; } /* > sqrt 2 */
  float f = m - 1.0f;                                           /* exact */
  float p = f32_from_bits(cb[8]);
  for (int i = 7; i >= 0; --i) p = fmaf(p, f, f32_from_bits(cb[i]));
  return fmaf((float)e, f32_from_bits(0x3F317218u), p * f);
}

/* The two standard normals of one 32-bit word, fp32, in this order of operations:
 *   L = -2 * ln(u1);  r = sqrt(L) (correctly rounded);
 *   angle 2 pi u2 = q * pi/2 + pi/4 + t with q = top 2 bits of the high half, j = its low 14 bits,
 *   t = (2 j + 1 - 16384) * fl(pi / 65536) in (-pi/4, pi/4);
 *   sin t = t + (t * t2) * S(t2), cos t = 1 + t2 * C(t2), t2 = t * t (S degree 2, C degree 3, Horner, fma);
 *   (c, s) = ((cos t - sin t) * fl(1/sqrt2), (cos t + sin t) * fl(1/sqrt2)), rotated by q quarter turns;
 *   z = (r * c, r * s).                                                                             */
void gwso_box_muller(uint32_t word, float z[2]) {
  float u1 = ((float)(word & 0xFFFFu) + 0.5f) * f32_from_bits(0x37800000u); /* 2^-16; exact */
  float L = -2.0f * bm_log(u1);
  float r = sqrtf(L);
  uint32_t hi = word >> 16, q = hi >> 14, j = hi & 0x3FFFu;
  float t = (float)(2 * (int)j + 1 - 16384) * f32_from_bits(0x38490FDBu);
  float t2 = t * t;
  float sp = f32_from_bits(0xB94D6501u);
  sp = fmaf(sp, t2, f32_from_bits(0x3C088615u));
  sp = fmaf(sp, t2, f32_from_bits(0xBE2AAAA9u));
  float st = fmaf(t * t2, sp, t);
  float cp = f32_from_bits(0x37CD3809u);
  cp = fmaf(cp, t2, f32_from_bits(0xBAB60706u));
  cp = fmaf(cp, t2, f32_from_bits(0x3D2AAAA6u));
  cp = fmaf(cp, t2, f32_from_bits(0xBF000000u));
  float ct = fmaf(t2, cp, 1.0f);
  float h = f32_from_bits(0x3F3504F3u);
  float c = (ct - st) * h, sn = (ct + st) * h;
  float cq, sq;
  switch (q) {
    case 0: cq = c; sq = sn; break;
    case 1: cq = -sn; sq = c; break;
    case 2: cq = -c; sq = -sn; break;
    default: cq = sn; sq = -c; break;
  }
  z[0] = r * cq;
  z[1] = r * sq;
}

void gwso_box_muller_n(const uint32_t* words, float* z, int64_t n) {
  for (int64_t i = 0; i < n; ++i) gwso_box_muller(words[i], z + 2 * i);
}

/* R of element k (= j & 7) of a group under a basis, from the group's four Philox words.
 *   *r16  : R as a BF16 bit pattern (bits basis and Box-Muller: 0, +-1, +-2, with the sign bit kept on a zero)
 * Returns R as a double (the value of *r16).                                                    */
double gwso_basis_r(const uint32_t x[4], int k, int basis, uint16_t* r16) {
  uint16_t out;
  if (basis == GWSO_BASIS_UNIFORM) {
    out = gwso_uniform_bf16((x[k >> 2] >> (8 * (k & 3))) & 0xFFu);
  } else {
    int mag, neg;
    if (basis == GWSO_BASIS_BOX_MULLER) {
      float z[2];
      gwso_box_muller(x[k >> 1], z);
      float rr = rintf(0.5f * z[k & 1]);           /* ties to even */
      neg = signbit(rr) ? 1 : 0;
      mag = (int)fabsf(rr);                        /* 0, 1 or 2: |z| < 4.86 with 16-bit u1 */
    } else {
      int code = element_code(x, k);
      mag = code & 3;
      neg = (code >> 3) & 1;
    }
    out = (uint16_t)((mag == 0 ? 0x0000u : (mag == 1 ? 0x3F80u : 0x4000u)) | (neg ? 0x8000u : 0u));
  }
  if (r16) *r16 = out;
  return (double)bf16_to_f32(out);
}

/* R of a whole [rows x cols] tensor under a basis, as fp32 (for the statistics pins). */
void gwso_noise_basis(int64_t rows, int64_t cols, int64_t row0, int64_t col0, uint64_t seed,
                      uint64_t step, int basis, float* r) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t j = 0; j < cols; ++j) {
      uint32_t x[4];
      group_words(row0 + i, (col0 + j) >> 3, seed, step, x);
      r[i * cols + j] = (float)gwso_basis_r(x, (int)((col0 + j) & 7), basis, NULL);
    }
}

/* ------------------------------------------------------------------ */
/* Forward, Eq. 3 + cast, one tensor.                                   */
/*   w, w_hat : BF16 [rows x cols], leading dimension ld (elements)     */
/*   bt       : fp32 [ceil(rows/32) x ceil(cols/32)]                    */
/*   scale    : out fp32 per block, s32 = max|w| * 2^(1-b_t) (unrounded */
/*              fp32; Eq. 4 reuses it)                                   */
/*   row0,col0: position inside a larger tensor (multiples of 32)       */
/* ------------------------------------------------------------------ */
static int sample_fwd_impl(const uint16_t* w, int64_t rows, int64_t cols, int64_t ld,
                           int64_t row0, int64_t col0, const float* bt, int fmt, int basis,
                           uint64_t seed, uint64_t step, uint16_t* w_hat, float* scale) {
  if (!w || !bt || !w_hat || !scale) return 1;
  if (fmt < 0 || fmt > 2 || basis < 0 || basis > 2) return 4;
  int64_t nbr = (rows + GWSO_BL - 1) / GWSO_BL, nbc = (cols + GWSO_BL - 1) / GWSO_BL;
#pragma omp parallel for schedule(static)
  for (int64_t bi = 0; bi < nbr; ++bi) {
    for (int64_t bj = 0; bj < nbc; ++bj) {
      int64_t i0 = bi * GWSO_BL, j0 = bj * GWSO_BL;
      int64_t i1 = i0 + GWSO_BL < rows ? i0 + GWSO_BL : rows;
      int64_t j1 = j0 + GWSO_BL < cols ? j0 + GWSO_BL : cols;
      /* max_{b_l}(|w|): exact, on the magnitude bits */
      uint16_t a16 = 0;
      for (int64_t i = i0; i < i1; ++i)
        for (int64_t j = j0; j < j1; ++j) {
          uint16_t mag = w[i * ld + j] & 0x7FFFu;
          if (mag > a16) a16 = mag;
        }
      /* scale = max|w| * 2^(1-b_t): fp32, then one rounding to BF16 */
      float t = 1.0f - bt[bi * nbc + bj];
      float p = gwso_exp2(t);
      float s32 = bf16_to_f32(a16) * p;
      uint16_t s16 = gwso_bf16_rne(s32);
      scale[bi * nbc + bj] = s32;
      int Ea = a16 ? floor_log2_bf16(a16) : 0;
      /* 2*s as a BF16 pattern (exact: exponent + 1), for |R| = 2 */
      uint16_t s2_16 = gwso_bf16_rne(2.0f * bf16_to_f32(s16));
      for (int64_t i = i0; i < i1; ++i) {
        for (int64_t j = j0; j < j1; ++j) {
          uint32_t x[4];
          /* recomputed per element: plain, not fast */
          group_words(row0 + i, (col0 + j) >> 3, seed, step, x);
          int code = element_code(x, (int)(j & 7));
          int mag = code & 3;
          /* PQN = R * s in sign-magnitude form: the sign bit is placed as is,
           * so R = "-0" gives -0.0 (Sec. 3.4: sign-mantissa reconstruction) */
          uint16_t pqn = (uint16_t)((mag == 0 ? 0u : (mag == 1 ? s16 : s2_16)) |
                                    ((code & 8) ? 0x8000u : 0u));
          if (basis != GWSO_BASIS_BITS) {
            /* another basis: PQN = bf16(R * s), which is exact for R in {0, +-1, +-2} */
            uint16_t r16;
            gwso_basis_r(x, (int)(j & 7), basis, &r16);
            pqn = gwso_bf16_mul(r16, s16);
          }
          uint16_t sum = gwso_bf16_add(w[i * ld + j], pqn);
          w_hat[i * ld + j] = (a16 == 0) ? sum : gwso_cast(sum, Ea, fmt);
        }
      }
    }
  }
  return 0;
}

int gwso_sample_fwd(const uint16_t* w, int64_t rows, int64_t cols, int64_t ld,
                    int64_t row0, int64_t col0, const float* bt, int fmt,
                    uint64_t seed, uint64_t step, uint16_t* w_hat, float* scale) {
  return sample_fwd_impl(w, rows, cols, ld, row0, col0, bt, fmt, GWSO_BASIS_BITS, seed, step, w_hat, scale);
}

/* The same forward pass with R drawn from another basis (see the bases above). */
int gwso_sample_fwd_basis(const uint16_t* w, int64_t rows, int64_t cols, int64_t ld,
                          int64_t row0, int64_t col0, const float* bt, int fmt, int basis,
                          uint64_t seed, uint64_t step, uint16_t* w_hat, float* scale) {
  return sample_fwd_impl(w, rows, cols, ld, row0, col0, bt, fmt, basis, seed, step, w_hat, scale);
}

/* ------------------------------------------------------------------ */
/* Backward, Eq. 4, one tensor.                                         */
/*   g   : dL/dw_hat, BF16                                              */
/*   dw  : out, = g bit for bit (may be NULL)                           */
/*   dbt : out fp64 per block, -ln2 * s32 * sum(g .* R)                 */
/*   abs_sum : out fp64 per block (may be NULL), ln2 * s32 * sum|g .* R|,*/
/*             the scale of rounding error a fp32 reduction may show     */
/* ------------------------------------------------------------------ */
static int sample_bwd_impl(const uint16_t* g, int64_t rows, int64_t cols, int64_t ld,
                           int64_t row0, int64_t col0, const float* scale, int basis, uint64_t seed,
                           uint64_t step, uint16_t* dw, double* dbt, double* abs_sum) {
  if (!g || !scale || !dbt) return 1;
  if (basis < 0 || basis > 2) return 4;
  int64_t nbr = (rows + GWSO_BL - 1) / GWSO_BL, nbc = (cols + GWSO_BL - 1) / GWSO_BL;
  const double ln2 = 0.69314718055994530942;
#pragma omp parallel for schedule(static)
  for (int64_t bi = 0; bi < nbr; ++bi) {
    for (int64_t bj = 0; bj < nbc; ++bj) {
      int64_t i0 = bi * GWSO_BL, j0 = bj * GWSO_BL;
      int64_t i1 = i0 + GWSO_BL < rows ? i0 + GWSO_BL : rows;
      int64_t j1 = j0 + GWSO_BL < cols ? j0 + GWSO_BL : cols;
      double acc = 0.0, aacc = 0.0;
      for (int64_t i = i0; i < i1; ++i)
        for (int64_t j = j0; j < j1; ++j) {
          uint32_t x[4];
          group_words(row0 + i, (col0 + j) >> 3, seed, step, x);
          double r = (double)gwso_code_to_r(element_code(x, (int)(j & 7)));
          if (basis != GWSO_BASIS_BITS) r = gwso_basis_r(x, (int)(j & 7), basis, NULL);
          double term = (double)bf16_to_f32(g[i * ld + j]) * r;
          acc += term;
          aacc += fabs(term);
          if (dw) dw[i * ld + j] = g[i * ld + j];
        }
      double s = (double)scale[bi * nbc + bj];
      dbt[bi * nbc + bj] = -ln2 * s * acc;
      if (abs_sum) abs_sum[bi * nbc + bj] = ln2 * s * aacc;
    }
  }
  return 0;
}

int gwso_sample_bwd(const uint16_t* g, int64_t rows, int64_t cols, int64_t ld,
                    int64_t row0, int64_t col0, const float* scale, uint64_t seed,
                    uint64_t step, uint16_t* dw, double* dbt, double* abs_sum) {
  return sample_bwd_impl(g, rows, cols, ld, row0, col0, scale, GWSO_BASIS_BITS, seed, step, dw, dbt, abs_sum);
}

/* Eq. 4 with R drawn from another basis. */
int gwso_sample_bwd_basis(const uint16_t* g, int64_t rows, int64_t cols, int64_t ld,
                          int64_t row0, int64_t col0, const float* scale, int basis, uint64_t seed,
                          uint64_t step, uint16_t* dw, double* dbt, double* abs_sum) {
  return sample_bwd_impl(g, rows, cols, ld, row0, col0, scale, basis, seed, step, dw, dbt, abs_sum);
}

/* ------------------------------------------------------------------ */
/* The sampled weight as microscaling (MX) data: the deployment format  */
/* the paper targets (Sec. 3.1: MXFP; square blocks, so W and its        */
/* transpose share the bytes).  Per 32x32 block one E8M0 scale byte,     */
/* the biased exponent of X = 2^(Ea + 1 - emax), and per element the     */
/* code of q / X in the element format (OCP MX: FP8 E4M3, bias 7, no     */
/* Inf, S.1111.111 = NaN never produced; FP6 E3M2, bias 3, no NaN/Inf).  */
/* q is the value gwso_sample_fwd stores in its BF16 container.          */
/* ------------------------------------------------------------------ */

/* Value of an element code, by the format's definition. */
double gwso_mx_code_value(int code, int fmt) {
  int emax, emin, m;
  double maxv;
  fmt_params(fmt, &emax, &emin, &m, &maxv);
  int ebits = (fmt == GWSO_FMT_FP8_E4M3) ? 4 : 3;
  int mant = code & ((1 << m) - 1);
  int E = (code >> m) & ((1 << ebits) - 1);
  int sign = (code >> (m + ebits)) & 1;
  int bias = 1 - emin;
  double mag = E == 0 ? ldexp((double)mant, emin - m)
                      : ldexp(1.0 + (double)mant / (double)(1 << m), E - bias);
  return sign ? -mag : mag;
}

/* Code of a BF16 value that is a member of X * format: found by running
 * through the format's codes (0xFF if the value is not a member). */
int gwso_mx_encode(uint16_t q16, int Ea, int fmt) {
  int emax, emin, m;
  double maxv;
  fmt_params(fmt, &emax, &emin, &m, &maxv);
  int ebits = (fmt == GWSO_FMT_FP8_E4M3) ? 4 : 3;
  int nmag = 1 << (m + ebits);
  double y = fabs(ldexp((double)bf16_to_f32(q16), -(Ea + 1 - emax)));
  for (int c = 0; c < nmag; ++c) {
    if (fmt == GWSO_FMT_FP8_E4M3 && c == 0x7F) continue; /* NaN */
    if (gwso_mx_code_value(c, fmt) == y) return c | ((q16 & 0x8000u) ? nmag : 0);
  }
  return 0xFF;
}

/* Forward pass with MX output.
 *   codes  : FP8: one byte per element, row stride ldc bytes.
 *            FP6: element j of a row occupies bits [6j, 6j+6) of the row's
 *            bytes read as a little-endian bit string (8 elements = 6 bytes);
 *            unused bits of the last byte touched are 0.
 *   xscale : [nbr x nbc] bytes, Ea + 1 - emax + 127 (127 for an all-zero block)
 *   scale  : s32 as in gwso_sample_fwd                                        */
int gwso_sample_fwd_mx(const uint16_t* w, int64_t rows, int64_t cols, int64_t ld,
                       int64_t row0, int64_t col0, const float* bt, int fmt,
                       uint64_t seed, uint64_t step, uint8_t* codes, int64_t ldc,
                       uint8_t* xscale, float* scale) {
  if (!w || !bt || !codes || !xscale || !scale) return 1;
  if (fmt != GWSO_FMT_FP8_E4M3 && fmt != GWSO_FMT_FP6_E3M2) return 4;
  uint16_t* q = (uint16_t*)malloc((size_t)(rows > 0 ? rows : 1) * (size_t)ld * sizeof(uint16_t));
  if (!q) return 5;
  int rc = gwso_sample_fwd(w, rows, cols, ld, row0, col0, bt, fmt, seed, step, q, scale);
  if (rc) { free(q); return rc; }
  int emax, emin, m;
  double maxv;
  fmt_params(fmt, &emax, &emin, &m, &maxv);
  int64_t nbr = (rows + GWSO_BL - 1) / GWSO_BL, nbc = (cols + GWSO_BL - 1) / GWSO_BL;
  /* block scales: Ea = floor(log2 max|w|) from the block maximum, the plain way */
  for (int64_t bi = 0; bi < nbr; ++bi)
    for (int64_t bj = 0; bj < nbc; ++bj) {
      int64_t i0 = bi * GWSO_BL, j0 = bj * GWSO_BL;
      int64_t i1 = i0 + GWSO_BL < rows ? i0 + GWSO_BL : rows;
      int64_t j1 = j0 + GWSO_BL < cols ? j0 + GWSO_BL : cols;
      uint16_t a16 = 0;
      for (int64_t i = i0; i < i1; ++i)
        for (int64_t j = j0; j < j1; ++j) {
          uint16_t mag = w[i * ld + j] & 0x7FFFu;
          if (mag > a16) a16 = mag;
        }
      int Ea = a16 ? floor_log2_bf16(a16) : emax - 1;   /* all-zero block: X = 1 */
      xscale[bi * nbc + bj] = (uint8_t)(Ea + 1 - emax + 127);
    }
  int64_t row_bytes = fmt == GWSO_FMT_FP8_E4M3 ? cols : (cols * 6 + 7) / 8;
  for (int64_t i = 0; i < rows; ++i) {
    memset(codes + i * ldc, 0, (size_t)row_bytes);
    for (int64_t j = 0; j < cols; ++j) {
      int Ea = (int)xscale[(i / GWSO_BL) * nbc + j / GWSO_BL] - 127 - 1 + emax;
      int code = gwso_mx_encode(q[i * ld + j], Ea, fmt);
      if (fmt == GWSO_FMT_FP8_E4M3) {
        codes[i * ldc + j] = (uint8_t)code;
      } else {
        for (int b = 0; b < 6; ++b) {
          int64_t bit = 6 * j + b;
          if ((code >> b) & 1) codes[i * ldc + bit / 8] |= (uint8_t)(1u << (bit % 8));
        }
      }
    }
  }
  free(q);
  return 0;
}

/* ------------------------------------------------------------------ */
/* Bitwidth parametrisation (Sec. 3.6 "Bitwidth", Eq. 11 and Eq. 12).   */
/*   b_t = b_target + b_i * (b_init - b_target), per block, in fp32:    */
/*   the difference, the product and the sum are each rounded once, in  */
/*   the order the equation is written.                                 */
/* ------------------------------------------------------------------ */
void gwso_bitwidth(const float* bi, int64_t n, float b_init, float b_target, float* bt) {
  float delta = b_init - b_target;
  for (int64_t k = 0; k < n; ++k) {
    float prod = bi[k] * delta;
    bt[k] = b_target + prod;
  }
}

/* Gradient of L' = L + lambda * sum_layers( sum_blocks |b_t - b_target| / m )  */
/* (Eq. 12) with respect to b_i, for the n blocks handed in, which belong to a  */
/* layer of m blocks:                                                           */
/*   dL'/db_i = (b_init - b_target) * ( dL/db_t + (lambda / m) * sgn(b_t - b_target) ) */
/* sgn is taken on the fp32 b_t the forward pass used (sgn(0) = 0); everything  */
/* else is fp64.                                                                */
void gwso_bitwidth_grad(const float* bi, const double* dbt, int64_t n, float b_init,
                        float b_target, double lambda, int64_t m, double* dbi) {
  float delta = b_init - b_target;
  for (int64_t k = 0; k < n; ++k) {
    float prod = bi[k] * delta;
    float bt = b_target + prod;
    double sgn = bt > b_target ? 1.0 : (bt < b_target ? -1.0 : 0.0);
    dbi[k] = (double)delta * (dbt[k] + lambda / (double)m * sgn);
  }
}

/* ------------------------------------------------------------------ */
/* Linear forward with an already-sampled weight (Sec. 3.5: the matmul  */
/* consumes w_hat; BF16 inputs, wide accumulation, Sec. 4).             */
/*   x : BF16 [M x K] (ldx);  q : BF16 w_hat, [K x N] (ldq) or, when    */
/*   w_is_nk, [N x K];  rows_sel : optional list of nsel row indices of  */
/*   X to compute (NULL = all M rows).                                   */
/*   y64 : out fp64 [nsel x N] exact-ish sums; yabs : out fp64, sum of   */
/*   |x*q| per output (error scale); y16 : out BF16 of y64 (may be NULL) */
/* ------------------------------------------------------------------ */
static uint16_t bf16_from_double(double d) {
  /* fp64 -> BF16 with one RNE: round on the fp64 bit pattern */
  uint64_t u;
  memcpy(&u, &d, 8);
  uint64_t sign = u >> 63;
  int e = (int)((u >> 52) & 0x7FF);
  uint64_t man = u & 0xFFFFFFFFFFFFFull;
  if (e == 0 && man == 0) return (uint16_t)(sign << 15);
  int E = e - 1023;                       /* fp64 normal assumed (sums of BF16 products) */
  uint64_t sig = man | (1ull << 52);      /* 53-bit significand */
  int drop = 45;                          /* keep 8 bits */
  if (E < -126) drop += (-126 - E);       /* BF16 subnormal */
  if (drop > 60) return (uint16_t)(sign << 15);
  uint64_t keep = sig >> drop, rem = sig & ((1ull << drop) - 1), half = 1ull << (drop - 1);
  if (rem > half || (rem == half && (keep & 1))) keep += 1;
  int ef = (E < -126) ? 0 : E + 127;
  uint32_t field;
  if (E < -126) field = (uint32_t)keep;   /* may carry into the lowest normal: still right */
  else {
    if (keep >= 0x100u) { keep >>= 1; ef += 1; }
    field = ((uint32_t)ef << 7) | (uint32_t)(keep & 0x7F);
    if (ef >= 0xFF) field = 0x7F80u;
  }
  return (uint16_t)((sign << 15) | field);
}

int gwso_linear_fwd(const uint16_t* x, int64_t M, int64_t K, int64_t ldx,
                    const uint16_t* q, int64_t N, int64_t ldq, int w_is_nk,
                    const int64_t* rows_sel, int64_t nsel,
                    double* y64, double* yabs, uint16_t* y16) {
  if (!x || !q || !y64) return 1;
  int64_t R = rows_sel ? nsel : M;
#pragma omp parallel for schedule(static)
  for (int64_t rr = 0; rr < R; ++rr) {
    int64_t mrow = rows_sel ? rows_sel[rr] : rr;
    for (int64_t n = 0; n < N; ++n) {
      double acc = 0.0, aacc = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        double xv = (double)bf16_to_f32(x[mrow * ldx + k]);
        double qv = (double)bf16_to_f32(w_is_nk ? q[n * ldq + k] : q[k * ldq + n]);
        acc += xv * qv;
        aacc += fabs(xv * qv);
      }
      y64[rr * N + n] = acc;
      if (yabs) yabs[rr * N + n] = aacc;
      if (y16) y16[rr * N + n] = bf16_from_double(acc);
    }
  }
  return 0;
}
