// Wavefront-tile building blocks of the forward pass (paper Eq. 3 + cast), shared by
// the elementwise kernel and the sampling prologue of the fused linear.
// Internal to csrc/.
#pragma once

#include "gws_launch.h"

namespace gws {

// Valid elements of the 16-byte group at (row, col): 8, fewer at a ragged right
// edge, 0 outside.
__device__ __forceinline__ int valid_count(uint32_t row, uint32_t col, uint32_t rows, uint32_t cols) {
  if (row >= rows || col >= cols) return 0;
  const uint32_t left = cols - col;
  return left >= 8 ? 8 : (int)left;
}

__device__ __forceinline__ u32x4 load16(const GWS_GLOBAL uint16_t* p) {
  return __builtin_nontemporal_load((const GWS_GLOBAL u32x4*)p);
}
__device__ __forceinline__ void store16(GWS_GLOBAL uint16_t* p, const u32x4 v) {
  __builtin_nontemporal_store(v, (GWS_GLOBAL u32x4*)p);
}

// Zero the elements of a group that lie past the right edge (nv valid of 8).
__device__ __forceinline__ u32x4 mask_group(u32x4 v, int nv) {
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (k >= nv) v[k >> 1] &= (k & 1) ? 0x0000FFFFu : 0xFFFF0000u;
  return v;
}

__device__ __forceinline__ void store_partial(GWS_GLOBAL uint16_t* dst, const u32x4 v, int nv) {
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (k < nv) dst[k] = (uint16_t)(v[k >> 1] >> ((k & 1) * 16));
}

// The four 16-byte groups a lane holds of one wavefront tile.
struct Tile {
  u32x4 v[4];
  int nv[4];   // valid elements per group (8 everywhere on a full tile)
  bool full;   // the 32x64 tile lies inside the tensor: no validity tests needed
};

// A 16-byte load never leaves its row: ld % 8 == 0 and ld >= cols.
__device__ __forceinline__ Tile load_tile(const GWS_GLOBAL uint16_t* __restrict__ src, const TileDesc& d, uint32_t by,
                                          uint32_t col_base, uint32_t col, uint32_t r0) {
  Tile t;
  const uint32_t row_base = by * 32;
  t.full = (row_base + 32 <= d.rows) && (col_base + 64 <= d.cols);
  if (t.full) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      t.nv[i] = 8;
      t.v[i] = load16(src + (size_t)(row_base + r0 + 8 * i) * d.ld + col);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t row = row_base + r0 + 8 * i;
      t.nv[i] = valid_count(row, col, d.rows, d.cols);
      t.v[i] = u32x4{0, 0, 0, 0};
      if (t.nv[i] > 0) t.v[i] = load16(src + (size_t)row * d.ld + col);
    }
  }
  return t;
}

// Element codes of one group to memory.  FP8: 8 bytes at column col.  FP6: 6 bytes at
// (col / 8) * 6, written as three 2-byte stores (a row of codes is only 2-byte aligned).
// nv < 8: only the bytes that hold existing elements (unused bits of the last one are 0).
template <int FMT>
__device__ __forceinline__ void store_codes(GWS_GLOBAL uint8_t* row, uint32_t col, const MxCodes c, int nv) {
  if (FMT == 1) {
    GWS_GLOBAL uint8_t* dst = row + col;
    if (nv == 8) {
      typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
      __builtin_nontemporal_store(u32x2{c.lo, c.hi}, (GWS_GLOBAL u32x2*)dst);
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k < nv) dst[k] = (uint8_t)((k < 4 ? c.lo : c.hi) >> (8 * (k & 3)));
    }
  } else {
    GWS_GLOBAL uint8_t* dst = row + (col >> 3) * 6;
    if (nv == 8) {
      GWS_GLOBAL uint16_t* d16 = (GWS_GLOBAL uint16_t*)dst;
      __builtin_nontemporal_store((uint16_t)c.lo, d16);
      __builtin_nontemporal_store((uint16_t)(c.lo >> 16), d16 + 1);
      __builtin_nontemporal_store((uint16_t)c.hi, d16 + 2);
    } else {
      // the fields of elements past the edge hold noise: clear them
      const uint64_t bits = (((uint64_t)c.hi << 32) | c.lo) & (((uint64_t)1 << (6 * nv)) - 1);
      const int nbytes = (nv * 6 + 7) >> 3;
#pragma unroll
      for (int k = 0; k < 6; ++k)
        if (k < nbytes) dst[k] = (uint8_t)(bits >> (8 * k));
    }
  }
}

// The forward pass on one wavefront tile, in two phases.
//
// tile_scale: a = max|w| of the lane's block (exact), the block's scale and cast constants.
//   BT_PRE: the caller has already fetched this lane's block parameter (bt_pre), as a wavefront that works
//   through several tiles alone does together with the tile loads, so that its latency is not paid per tile.
//   STORE: the block's writer lane stores scale (and, MX, the E8M0 block scale) here; off, the caller does.
// tile_apply: noise, add, round, cast, store.
//   STREAM: w_hat is written with streaming (non-temporal) stores, right for a pass that is not consumed at
//   once; off, the stores stay in cache for a reader that follows.
//   MX: the output is element codes (p1, row stride ldc) and E8M0 block scales (p4) instead of the BF16 container.
//   BASIS: kBasisBits is the method's noise (Sec. 3.4); the other two are the comparison bases (no MX form).
//   USE_HW: FP8-E4M3 through the hardware converters (the caller has shown that no block of the wavefront can
//   overflow); off, the arithmetic cast.  Same bits either way where both apply.
//   rows_part: the row-only share of the lane's four Philox calls, when the caller keeps it across column tiles
//   (philox_rows of the rows d.row0 + 32 by + lane / 8 + 8 i); bits: the four calls' results themselves, when
//   the caller has them already; both NULL: every call is computed on its own.
// Neither phase branches when FULL and !STORE, so a caller that works on several tiles at once gets straight-line
// code it can interleave.
template <int FMT, bool FULL, bool MX, bool BT_PRE, bool STORE>
__device__ __forceinline__ BlockScale tile_scale(const TileDesc& d, Tile& t, uint32_t by, uint32_t col_base, uint32_t lane,
                                                 float bt_pre) {
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  const GWS_GLOBAL float* __restrict__ bt = global_ptr<float>(d.p2);
  GWS_GLOBAL float* __restrict__ scale = global_ptr<float>(d.p3);
  if (!FULL) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (t.nv[i] < 8) t.v[i] = mask_group(t.v[i], t.nv[i]);  // elements past cols do not exist
  }
  // ---- a = max_{b_l}|w| on the magnitude bits (exact) ----
  uint32_t m = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) m = absmax_pk(t.v[i], m);
  m = max(m & 0xFFFFu, m >> 16);
  const uint32_t a16 = block_max_u32(m);
  // ---- per-block scale ----
  const uint32_t nbc = (d.cols + 31) >> 5;
  const uint32_t bcol = (col_base >> 5) + (gc >> 2);
  const bool block_exists = FULL || bcol < nbc;
  const float bv = BT_PRE ? bt_pre : (block_exists ? bt[(size_t)by * nbc + bcol] : 0.0f);
  // Eq. 11 (the product and the sum rounded separately); identity for a plain b_t
  const float btv = __fadd_rn(d.b_target, __fmul_rn(bv, d.b_delta));
  BlockScale b = block_scale(a16, btv);
  if (FMT == 1) cast_constants<8, -6>(a16, b);
  if (FMT == 2) cast_constants<4, -2>(a16, b);
  if (STORE && block_exists && (gc & 3) == 0 && r0 == 0) {
    scale[(size_t)by * nbc + bcol] = b.s32;
    // shared exponent of the block: biased exponent of X; X = 1 for an all-zero block
    if (MX) global_ptr<uint8_t>(d.p4)[(size_t)by * nbc + bcol] = a16 ? (uint8_t)(__float_as_uint(b.x_scale) >> 23) : (uint8_t)127;
  }
  return b;
}

template <int FMT, bool FULL, bool STREAM, bool MX, int BASIS, bool USE_HW>
__device__ __forceinline__ void tile_apply(uint32_t step_lo, uint32_t step_hi, const TileDesc& d, const Tile& t,
                                           const BlockScale& b, uint32_t by, uint32_t col_base, uint32_t lane,
                                           const PhiloxRows* rows_part, const Philox4* bits) {
  static_assert(BASIS == kBasisBits || !MX, "the comparison bases have no MX output");
  static_assert(!USE_HW || FMT == 1, "hardware converters by choice exist for FP8-E4M3 only");
  const uint32_t row_base = by * 32;
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  const uint32_t col = col_base + gc * 8;
  GWS_GLOBAL uint16_t* __restrict__ w_hat = global_ptr<uint16_t>(d.p1);
  const uint32_t cg = d.cg0 + (col >> 3);
  PhiloxCols pc = {};
  if (bits == nullptr && rows_part != nullptr) pc = philox_cols(cg, step_lo, step_hi, d.seed_lo, d.seed_hi);
  auto bits_of = [&](uint32_t row, int i) {   // the 128 bits of the lane's group i (row = its global row)
    return bits != nullptr         ? bits[i]
           : rows_part != nullptr ? philox_row(pc, *rows_part, i, d.seed_lo, d.seed_hi)
                                   : philox4x32_10(cg, row, step_lo, step_hi, d.seed_lo, d.seed_hi);
  };
  // the four BF16 sums of group i (before the cast), whatever the basis
  auto sampled_group = [&](const u32x4 w, uint32_t row, int i, uint32_t (&pk)[4]) {
    if constexpr (BASIS == kBasisBits) {
      const Noise n = noise_planes(bits_of(row, i));
      const GroupMagnitudes g = group_magnitudes(n);
      pk[0] = sampled_pair<0>(w[0], g, n, b);
      pk[1] = sampled_pair<1>(w[1], g, n, b);
      pk[2] = sampled_pair<2>(w[2], g, n, b);
      pk[3] = sampled_pair<3>(w[3], g, n, b);
    } else {
      const Philox4 x = bits_of(row, i);
      pk[0] = sampled_pair_basis<BASIS, 0>(w[0], x, b);
      pk[1] = sampled_pair_basis<BASIS, 1>(w[1], x, b);
      pk[2] = sampled_pair_basis<BASIS, 2>(w[2], x, b);
      pk[3] = sampled_pair_basis<BASIS, 3>(w[3], x, b);
    }
  };
  if constexpr (FMT != 2) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (!FULL && t.nv[i] == 0) continue;
      const uint32_t row = row_base + r0 + 8 * i;
      if constexpr (MX) {
        const Noise n = noise_planes(bits_of(d.row0 + row, i));
        const MxCodes c = sample_group_mx_fp8(t.v[i], n, b, USE_HW);
        store_codes<FMT>(global_ptr<uint8_t>(d.p1) + (size_t)row * d.ldc, col, c, FULL ? 8 : t.nv[i]);
      } else {
        uint32_t pk[4];
        sampled_group(t.v[i], d.row0 + row, i, pk);
        i16x2 chain = {0, 0};
        const u32x4 o = {cast_pair<FMT>(pk[0], b, USE_HW, chain), cast_pair<FMT>(pk[1], b, USE_HW, chain),
                         cast_pair<FMT>(pk[2], b, USE_HW, chain), cast_pair<FMT>(pk[3], b, USE_HW, chain)};
        GWS_GLOBAL uint16_t* dst = w_hat + (size_t)row * d.ld + col;
        if (FULL || t.nv[i] == 8) {
          if (STREAM) store16(dst, o);
          else *(GWS_GLOBAL u32x4*)dst = o;
        } else {
          store_partial(dst, o, t.nv[i]);
        }
      }
    }
  } else {
    // FP6-E3M2: the 32-wide hardware converters (v_cvt_scalef32_pk32_bf6_bf16 and back) take
    // a lane's whole tile at once, round to nearest even with gradual underflow and saturate
    // at 28 * X (checked against the cast's definition on every finite BF16 input at several
    // scales), so all four groups are sampled first and converted together.
    typedef __bf16 bf16x32 __attribute__((ext_vector_type(32)));
    typedef uint32_t u32x6 __attribute__((ext_vector_type(6)));
    uint32_t pk[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (!FULL && t.nv[i] == 0) {
        pk[4 * i] = pk[4 * i + 1] = pk[4 * i + 2] = pk[4 * i + 3] = 0;
        continue;
      }
      uint32_t p4[4];
      sampled_group(t.v[i], d.row0 + row_base + r0 + 8 * i, i, p4);
      pk[4 * i] = p4[0];
      pk[4 * i + 1] = p4[1];
      pk[4 * i + 2] = p4[2];
      pk[4 * i + 3] = p4[3];
    }
    bf16x32 v;
    __builtin_memcpy(&v, pk, 64);
    const u32x6 c = __builtin_amdgcn_cvt_scalef32_pk32_bf6_bf16(v, b.x_scale);
    if constexpr (MX) {
      // element k of the lane's 32 sits in bits [6k, 6k + 6): 48 bits per group
      const MxCodes gc4[4] = {{c[0], c[1] & 0xFFFFu},
                              {(c[1] >> 16) | (c[2] << 16), c[2] >> 16},
                              {c[3], c[4] & 0xFFFFu},
                              {(c[4] >> 16) | (c[5] << 16), c[5] >> 16}};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (!FULL && t.nv[i] == 0) continue;
        const uint32_t row = row_base + r0 + 8 * i;
        store_codes<FMT>(global_ptr<uint8_t>(d.p1) + (size_t)row * d.ldc, col, gc4[i], FULL ? 8 : t.nv[i]);
      }
    } else {
      const bf16x32 q = __builtin_amdgcn_cvt_scalef32_pk32_bf16_bf6(c, b.x_scale);
      uint32_t o[16];
      __builtin_memcpy(o, &q, 64);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (!FULL && t.nv[i] == 0) continue;
        const uint32_t row = row_base + r0 + 8 * i;
        const u32x4 og = {o[4 * i], o[4 * i + 1], o[4 * i + 2], o[4 * i + 3]};
        GWS_GLOBAL uint16_t* dst = w_hat + (size_t)row * d.ld + col;
        if (FULL || t.nv[i] == 8) {
          if (STREAM) store16(dst, og);
          else *(GWS_GLOBAL u32x4*)dst = og;
        } else {
          store_partial(dst, og, t.nv[i]);
        }
      }
    }
  }
}

// Both phases for one tile; FP8-E4M3 takes the hardware converters only if neither block of this wavefront can
// overflow (they give NaN where the cast saturates).
template <int FMT, bool FULL, bool STREAM = true, bool MX = false, bool BT_PRE = false, int BASIS = kBasisBits>
__device__ __forceinline__ void fwd_tile(uint32_t step_lo, uint32_t step_hi, const TileDesc& d, Tile& t,
                                         uint32_t by, uint32_t col_base, uint32_t lane, float bt_pre = 0.0f,
                                         const PhiloxRows* rows_part = nullptr) {
  const BlockScale b = tile_scale<FMT, FULL, MX, BT_PRE, true>(d, t, by, col_base, lane, bt_pre);
  if constexpr (FMT == 1) {
    if (__builtin_amdgcn_ballot_w64(!b.hw_safe) == 0)
      tile_apply<FMT, FULL, STREAM, MX, BASIS, true>(step_lo, step_hi, d, t, b, by, col_base, lane, rows_part, nullptr);
    else
      tile_apply<FMT, FULL, STREAM, MX, BASIS, false>(step_lo, step_hi, d, t, b, by, col_base, lane, rows_part, nullptr);
  } else {
    tile_apply<FMT, FULL, STREAM, MX, BASIS, false>(step_lo, step_hi, d, t, b, by, col_base, lane, rows_part, nullptr);
  }
}

}  // namespace gws
