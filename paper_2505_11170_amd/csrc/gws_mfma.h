// Shared by the large-tile MFMA GEMM kernels (internal to csrc/).
#pragma once

#include "gws_launch.h"

namespace gws {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace g256 {
constexpr int TM = 256, TN = 256, TK = 64;
constexpr int PA = TK + 8;        // pitch of a tile kept contraction-contiguous, in elements (144 B)
constexpr int PB_KN = TN + 16;    // pitch of a tile kept output-contiguous, in elements (544 B)
constexpr int A_STAGE = TM * PA;                  // elements
constexpr int B_STAGE_NK = TN * PA;
constexpr int B_STAGE_KN = TK * PB_KN;
constexpr int PC = 128 + 8;       // epilogue pitch per wavefront tile (elements)
constexpr size_t lds_bytes(bool nk) {
  return (size_t)2 * (2 * A_STAGE + 2 * (nk ? B_STAGE_NK : B_STAGE_KN));
}
constexpr size_t lds_bytes_tn() { return (size_t)2 * (4 * B_STAGE_KN); }
}  // namespace g256

union Frag8 {
  u32x4 u;
  bf16x8 v;
  i16x4 h[2];
};

// XCD-aware tile numbering: launch-order number L -> (tile_m, tile_n) of an mt x nt grid of
// tiles.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2; XCD x gets
// a contiguous range of an order that walks 8 m-tiles down before moving one n-tile right,
// so the 32 workgroups running together on an XCD form an 8 x 4 patch sharing 8 + 4 panels.
__device__ __forceinline__ void tile_of(uint32_t L, uint32_t mt, uint32_t nt, uint32_t& tile_m, uint32_t& tile_n) {
  const uint32_t total = mt * nt;
  const uint32_t per = total / 8, rem = total % 8, x = L % 8, j = L / 8;
  L = x * per + (x < rem ? x : rem) + j;            // XCD x owns `per` tiles (+1 for the first `rem`)
  const uint32_t band_sz = 8 * nt;                   // tiles in a band of 8 m-tiles
  const uint32_t band = L / band_sz, r = L % band_sz;
  const uint32_t mrows = (band * 8 + 8 <= mt) ? 8 : (mt - band * 8);  // last band may be short
  tile_n = r / mrows;
  tile_m = band * 8 + r % mrows;
}

}  // namespace gws
