// Large-tile BF16 MFMA GEMM for gfx950: Y[M x N] = X[M x K] * W, W stored [K x N] or
// [N x K].  Used when M, N are multiples of 256 and K of 64.  The tile itself (direct
// global -> LDS loads, swizzled stages, pinned MFMA / LDS-read / load interleave) is in
// gws_gemm256_core.h; here are the plain kernel and the plain kernel with another weight's
// sampling riding at the end of its grid.
// Tiles are numbered so that the 32 workgroups running together on one XCD
// (workgroups are dealt round-robin to the 8 XCDs, each with its own L2) form an
// 8 x 4 patch that shares 8 X panels and 4 W panels.
#include "gws_gemm256_core.h"
#include "gws_launch.h"
#include "gws_sample_tile.h"

namespace gws {

// One 256 x 256 output tile.  `L` is the launch-order tile number, `wsrc` the weight
// operand (W, or the sampled w_hat).
template <bool W_NK>
__device__ __forceinline__ void gemm256_tile(const GemmArgs& g, const uint16_t* __restrict__ wsrc, uint32_t L) {
  uint32_t tile_m, tile_n;
  tile_of(L, g.M / g256::TM, g.N / g256::TN, tile_m, tile_n);
  gemm256_core<false, !W_NK>(g.x, g.ldx, wsrc, g.ldw, g.y, g.ldy, g.K / g256::TK, tile_m * g256::TM,
                             tile_n * g256::TN, NoHook{});
}

template <bool W_NK>
__global__ __launch_bounds__(256, 1) void gemm256_kernel(const GemmArgs g) {
  gemm256_tile<W_NK>(g, g.w, blockIdx.x);
}

// The stored weight seen as the forward kernel sees it: 32-row x 256-column
// workgroup tiles of four wavefront tiles (32 x 64, two blocks each).  Wavefront
// tile t covers block row t / (cols/64), columns 64 * (t % (cols/64)).  A batch of
// kDepth tiles is loaded before the first is computed, so the single wavefront per
// SIMD pays the memory latency once per batch; neighbouring wavefronts take
// neighbouring tiles, so a workgroup reads 512 contiguous bytes per row.
template <int FMT, int kDepth = 3>
__device__ __forceinline__ void sample_tiles(uint32_t step_lo, uint32_t step_hi, const TileDesc& d, uint32_t first,
                                             uint32_t stride, uint32_t lane) {
  const uint32_t per_row = d.cols >> 6, ntiles = (d.rows >> 5) * per_row;
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  for (uint32_t base = first; base < ntiles; base += kDepth * stride) {
    Tile t[kDepth];
    float bv[kDepth];   // the lane's block parameter, fetched with the tile instead of once the tile is reduced
#pragma unroll
    for (int j = 0; j < kDepth; ++j) {
      const uint32_t id = base + j * stride;
      if (id < ntiles) {
        const uint32_t by = id / per_row, cb = (id - by * per_row) * 64;
        t[j] = load_tile(global_ptr<uint16_t>(d.p0), d, by, cb, cb + gc * 8, r0);
        bv[j] = global_ptr<float>(d.p2)[(size_t)by * (d.cols >> 5) + (cb >> 5) + (gc >> 2)];
      }
    }
#pragma unroll
    for (int j = 0; j < kDepth; ++j) {
      const uint32_t id = base + j * stride;
      if (id < ntiles) {
        const uint32_t by = id / per_row, cb = (id - by * per_row) * 64;
        fwd_tile<FMT, true, false, false, true>(step_lo, step_hi, d, t[j], by, cb, lane, bv[j]);
      }
    }
  }
}

// The riding form of the sampling for weights of whole 32 x 256 tiles (up to kMaxRide of them, numbered through):
// a wavefront takes one such tile (four wavefront tiles side by side: 1 KiB contiguous per row, the same rows) per
// step and the grid's wavefronts take tiles round-robin.  A riding wavefront has its SIMD to itself and the GEMM's
// register allocation, so it keeps two tiles' worth of loads in flight (the next 32 x 256 tile is fetched before
// the current one is computed), and since nothing else hides its vector ALU latency the Philox rounds of two
// wavefront tiles are advanced together (philox_two_tiles) and the four wavefront tiles are straight-line code; the
// row-only rounds are shared by the four.
template <int FMT>
__device__ __forceinline__ void ride_tiles(uint32_t step_lo, uint32_t step_hi, const RideList& r, uint32_t first,
                                           uint32_t stride, uint32_t lane) {
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  const bool writer = (gc & 3) == 0 && r0 == 0;
  const uint32_t total = r.begin[kMaxRide];
  struct Batch {
    Tile t[4];
    float bv[4];
  };
  // which weight a tile number belongs to (uniform: tile numbers are per wavefront)
  auto weight_of = [&](uint32_t id) {
    uint32_t k = 0;
#pragma unroll
    for (int j = 1; j < kMaxRide; ++j) k += (id >= r.begin[j]) ? 1u : 0u;   // begin[] of unused entries = total
    return k;
  };
  auto fetch = [&](uint32_t id, Batch& b) {
    const TileDesc& d = r.d[weight_of(id)];
    const uint32_t local = id - d.first_wg, per_row = d.cols >> 8, nbc = d.cols >> 5;
    const uint32_t by = local / per_row, cb0 = (local - by * per_row) * 256;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      b.t[j] = load_tile(global_ptr<uint16_t>(d.p0), d, by, cb0 + 64 * j, cb0 + 64 * j + gc * 8, r0);
      b.bv[j] = global_ptr<float>(d.p2)[(size_t)by * nbc + ((cb0 + 64 * j) >> 5) + (gc >> 2)];
    }
  };
  if (first >= total) return;
  Batch cur;
  fetch(first, cur);
  for (uint32_t id = first; id < total; id += stride) {
    Batch nxt;
    const bool more = id + stride < total;   // uniform
    if (more) fetch(id + stride, nxt);
    const TileDesc& d = r.d[weight_of(id)];
    const uint32_t local = id - d.first_wg, per_row = d.cols >> 8, nbc = d.cols >> 5;
    const uint32_t by = local / per_row, cb0 = (local - by * per_row) * 256;
    uint32_t rows[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) rows[i] = d.row0 + by * 32 + r0 + 8 * i;
    const PhiloxRows rp = philox_rows(rows, step_lo, d.seed_lo);
    BlockScale bs[4];
    bool unsafe = false;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bs[j] = tile_scale<FMT, true, false, true, false>(d, cur.t[j], by, cb0 + 64 * j, lane, cur.bv[j]);
      unsafe |= !bs[j].hw_safe;
    }
    Philox4 bits[4][4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const PhiloxCols pc[2] = {philox_cols(d.cg0 + ((cb0 + 128 * h) >> 3) + gc, step_lo, step_hi, d.seed_lo, d.seed_hi),
                                philox_cols(d.cg0 + ((cb0 + 128 * h + 64) >> 3) + gc, step_lo, step_hi, d.seed_lo, d.seed_hi)};
      Philox4 two[2][4];
      philox_two_tiles(pc, rp, d.seed_lo, d.seed_hi, two);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bits[2 * h][i] = two[0][i];
        bits[2 * h + 1][i] = two[1][i];
      }
    }
    // FP8-E4M3: the hardware converters if no block of the four tiles can overflow
    if (FMT == 1 && __builtin_amdgcn_ballot_w64(unsafe) == 0) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        tile_apply<FMT, true, false, false, kBasisBits, FMT == 1>(step_lo, step_hi, d, cur.t[j], bs[j], by, cb0 + 64 * j, lane,
                                                                   &rp, bits[j]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        tile_apply<FMT, true, false, false, kBasisBits, false>(step_lo, step_hi, d, cur.t[j], bs[j], by, cb0 + 64 * j, lane,
                                                                &rp, bits[j]);
    }
    if (writer) {
      GWS_GLOBAL float* sc = global_ptr<float>(d.p3) + (size_t)by * nbc + (cb0 >> 5) + (gc >> 2);
#pragma unroll
      for (int j = 0; j < 4; ++j) sc[2 * j] = bs[j].s32;
    }
    if (more) cur = nxt;
  }
}

// Plain GEMM with the forward sampling of other weights riding along: the grid is the GEMM's tiles followed by
// `gridDim.x - tiles` more workgroups, which start when compute units run out of tiles (the last, partly empty
// round) and sample the weights of `r` while the last tiles finish.  The two halves share nothing: no
// synchronisation, no state.
// RIDER: 0 = sample_tiles on r.d[0] alone (any weight of whole 32 x 64 tiles), 1 = ride_tiles (whole 32 x 256 tiles)
template <int FMT, bool W_NK, int RIDER>
__global__ __launch_bounds__(256, 1) void gemm256_ride_kernel(const GemmArgs g, const RideList r, const uint32_t step_lo,
                                                              const uint32_t step_hi, const uint32_t tiles) {
  if (blockIdx.x < tiles) {
    gemm256_tile<W_NK>(g, g.w, blockIdx.x);
  } else {
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const uint32_t first = (blockIdx.x - tiles) * 4 + wave, stride = (gridDim.x - tiles) * 4;
    if (RIDER == 1) ride_tiles<FMT>(step_lo, step_hi, r, first, stride, lane);
    else sample_tiles<FMT, 4>(step_lo, step_hi, r.d[0], first, stride, lane);
  }
}

template <int FMT, int RIDER>
static int launch_ride_fmt(const GemmArgs& g, int w_is_nk, const RideList& r, uint32_t step_lo, uint32_t step_hi,
                           uint32_t tiles, uint32_t extra, hipStream_t s) {
  if (w_is_nk)
    hipLaunchKernelGGL((gemm256_ride_kernel<FMT, true, RIDER>), dim3(tiles + extra), dim3(256), 0, s, g, r, step_lo, step_hi, tiles);
  else
    hipLaunchKernelGGL((gemm256_ride_kernel<FMT, false, RIDER>), dim3(tiles + extra), dim3(256), 0, s, g, r, step_lo, step_hi, tiles);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

int launch_gemm256_ride(const GemmArgs& g, int w_is_nk, const RideList& r, int fmt, uint64_t step, uint32_t extra,
                        int rider, hipStream_t stream) {
  const uint64_t tiles = (uint64_t)(g.M / g256::TM) * (g.N / g256::TN);
  if (tiles + extra >= 0x7FFFFFFFull) return GWS_ERR_SHAPE;
  const uint32_t lo = (uint32_t)step, hi = (uint32_t)(step >> 32);
  if (rider == 1) {
    switch (fmt) {
      case GWS_FMT_BF16: return launch_ride_fmt<0, 1>(g, w_is_nk, r, lo, hi, (uint32_t)tiles, extra, stream);
      case GWS_FMT_FP8_E4M3: return launch_ride_fmt<1, 1>(g, w_is_nk, r, lo, hi, (uint32_t)tiles, extra, stream);
      case GWS_FMT_FP6_E3M2: return launch_ride_fmt<2, 1>(g, w_is_nk, r, lo, hi, (uint32_t)tiles, extra, stream);
      default: return GWS_ERR_FORMAT;
    }
  }
  switch (fmt) {
    case GWS_FMT_BF16: return launch_ride_fmt<0, 0>(g, w_is_nk, r, lo, hi, (uint32_t)tiles, extra, stream);
    case GWS_FMT_FP8_E4M3: return launch_ride_fmt<1, 0>(g, w_is_nk, r, lo, hi, (uint32_t)tiles, extra, stream);
    case GWS_FMT_FP6_E3M2: return launch_ride_fmt<2, 0>(g, w_is_nk, r, lo, hi, (uint32_t)tiles, extra, stream);
    default: return GWS_ERR_FORMAT;
  }
}

int compute_units() {
  static const int cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return n;
  }();
  return cus;
}

// The tile's direct loads address a lane as a scalar base plus a 32-bit byte offset of up to seven rows of the operand.
bool gemm256_applicable(const GemmArgs& g) {
  return g.M % g256::TM == 0 && g.N % g256::TN == 0 && g.K % g256::TK == 0 && g.M > 0 && g.N > 0 && g.K > 0 &&
         g.ldx < g256::kMaxLd && g.ldw < g256::kMaxLd;
}

int launch_gemm256(const GemmArgs& g, int w_is_nk, hipStream_t stream) {
  const uint64_t tiles = (uint64_t)(g.M / g256::TM) * (g.N / g256::TN);
  if (tiles >= 0x7FFFFFFFull) return GWS_ERR_SHAPE;
  if (w_is_nk) hipLaunchKernelGGL(gemm256_kernel<true>, dim3((uint32_t)tiles), dim3(256), 0, stream, g);
  else hipLaunchKernelGGL(gemm256_kernel<false>, dim3((uint32_t)tiles), dim3(256), 0, stream, g);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

}  // namespace gws
