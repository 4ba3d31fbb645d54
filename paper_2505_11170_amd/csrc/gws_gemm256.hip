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

// Plain GEMM with the forward sampling of another weight riding along: the grid is the GEMM's tiles
// followed by `gridDim.x - tiles` more workgroups, which start when compute units run out of tiles (the
// last, partly empty round) and sample the weight `d` (32 x 64 wavefront tiles, as above) while the last
// tiles finish.  The two halves share nothing: no synchronisation, no state.
template <int FMT, bool W_NK>
__global__ __launch_bounds__(256, 1) void gemm256_ride_kernel(const GemmArgs g, const TileDesc d, const uint32_t step_lo,
                                                              const uint32_t step_hi, const uint32_t tiles) {
  if (blockIdx.x < tiles) {
    gemm256_tile<W_NK>(g, g.w, blockIdx.x);
  } else {
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    sample_tiles<FMT, 8>(step_lo, step_hi, d, (blockIdx.x - tiles) * 4 + wave, (gridDim.x - tiles) * 4, lane);
  }
}

template <int FMT>
static int launch_ride_fmt(const GemmArgs& g, int w_is_nk, const TileDesc& d, uint32_t step_lo, uint32_t step_hi,
                           uint32_t tiles, uint32_t extra, hipStream_t s) {
  if (w_is_nk)
    hipLaunchKernelGGL((gemm256_ride_kernel<FMT, true>), dim3(tiles + extra), dim3(256), 0, s, g, d, step_lo, step_hi, tiles);
  else
    hipLaunchKernelGGL((gemm256_ride_kernel<FMT, false>), dim3(tiles + extra), dim3(256), 0, s, g, d, step_lo, step_hi, tiles);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

int launch_gemm256_ride(const GemmArgs& g, int w_is_nk, const TileDesc& d, int fmt, uint64_t step, uint32_t extra,
                        hipStream_t stream) {
  const uint64_t tiles = (uint64_t)(g.M / g256::TM) * (g.N / g256::TN);
  if (tiles + extra >= 0x7FFFFFFFull) return GWS_ERR_SHAPE;
  const uint32_t lo = (uint32_t)step, hi = (uint32_t)(step >> 32);
  switch (fmt) {
    case GWS_FMT_BF16: return launch_ride_fmt<0>(g, w_is_nk, d, lo, hi, (uint32_t)tiles, extra, stream);
    case GWS_FMT_FP8_E4M3: return launch_ride_fmt<1>(g, w_is_nk, d, lo, hi, (uint32_t)tiles, extra, stream);
    case GWS_FMT_FP6_E3M2: return launch_ride_fmt<2>(g, w_is_nk, d, lo, hi, (uint32_t)tiles, extra, stream);
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

bool gemm256_applicable(const GemmArgs& g) {
  return g.M % g256::TM == 0 && g.N % g256::TN == 0 && g.K % g256::TK == 0 && g.M > 0 && g.N > 0 && g.K > 0;
}

int launch_gemm256(const GemmArgs& g, int w_is_nk, hipStream_t stream) {
  const uint64_t tiles = (uint64_t)(g.M / g256::TM) * (g.N / g256::TN);
  if (tiles >= 0x7FFFFFFFull) return GWS_ERR_SHAPE;
  if (w_is_nk) hipLaunchKernelGGL(gemm256_kernel<true>, dim3((uint32_t)tiles), dim3(256), 0, stream, g);
  else hipLaunchKernelGGL(gemm256_kernel<false>, dim3((uint32_t)tiles), dim3(256), 0, stream, g);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

}  // namespace gws
