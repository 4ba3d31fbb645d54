// Large-tile BF16 MFMA GEMM for gfx950: Y[M x N] = X[M x K] * W, W stored [K x N] or
// [N x K].  Used when M, N are multiples of 256 and K of 64.  The tile itself (direct
// global -> LDS loads, swizzled stages, pinned MFMA / LDS-read / load interleave) is in
// gws_gemm256_core.h; here are the plain kernel, the fused sample-once kernel and the
// plain kernel with another weight's sampling riding at the end of its grid.
// Tiles are numbered so that the 32 workgroups running together on one XCD
// (workgroups are dealt round-robin to the 8 XCDs, each with its own L2) form an
// 8 x 4 patch that shares 8 X panels and 4 W panels.
#include <atomic>

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

// ---------------------------------------------------------------------------
// Fused sampled-weight linear, sample-once form.  A persistent grid (one
// workgroup per compute unit) first samples W cooperatively: every wavefront
// takes 32x64 tiles of the stored matrix round-robin (paper Eq. 3 + cast, as in
// the forward kernel), writes w_hat and scale, and the grid meets at one
// device-wide arrival counter.  The tiles of the GEMM then read w_hat through
// L2 like a plain weight.  Each block is sampled once, instead of once per
// M-tile as when the sampling sits in the operand load itself.
//
// Synchronisation state lives in a few device words.  The arrival counters reset
// themselves; the epoch and flag words are compared with a per-call epoch, so stale
// values of earlier calls never match.  The wait is bounded: a workgroup that gives up
// (e.g. because not all workgroups are resident) samples every block itself,
// which produces the same bytes.  Calls that overlap in time on one GPU would
// share the two words and must not be issued concurrently.
// ---------------------------------------------------------------------------
// Eight arrival groups (workgroup index mod 8: one per XCD when workgroups are dealt
// round-robin), each with its own counter and flag on its own 128-byte line, and one
// top-level counter for the eight group leaders.  Far fewer workgroups then contend for,
// and poll, any one address than with a single flat counter.
__device__ uint32_t g_fused_group_arrive[8 * 32];
__device__ uint32_t g_fused_group_flag[8 * 32];
__device__ uint32_t g_fused_top_arrive = 0;
__device__ uint32_t g_fused_epoch = 0;

// Returns true when every workgroup of the grid has arrived (and their earlier stores
// are visible), false when the bounded wait ran out.  Called by one thread per workgroup.
__device__ __forceinline__ bool grid_arrive_and_wait(uint32_t epoch) {
  const uint32_t grp = blockIdx.x & 7u;
  const uint32_t members = (gridDim.x >> 3) + ((grp < (gridDim.x & 7u)) ? 1u : 0u);
  const uint32_t groups = gridDim.x < 8u ? gridDim.x : 8u;
  __threadfence();  // release: this workgroup's w_hat / scale stores are visible device-wide
  uint32_t spins = 0;
  const uint32_t old = __hip_atomic_fetch_add(&g_fused_group_arrive[grp * 32], 1u, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
  if (old == members - 1) {  // last of its group: reset the counter, arrive at the top level
    __hip_atomic_store(&g_fused_group_arrive[grp * 32], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t t = __hip_atomic_fetch_add(&g_fused_top_arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == groups - 1) {
      __hip_atomic_store(&g_fused_top_arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&g_fused_epoch, epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
    // polls are relaxed loads (an acquire load would invalidate caches on every poll, under
    // the feet of the workgroups still sampling); one acquire fence follows the wait
    while (__hip_atomic_load(&g_fused_epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
      if (++spins > 200000u) return false;  // bounded wait (about 0.1 s)
      __builtin_amdgcn_s_sleep(4);
    }
    __hip_atomic_store(&g_fused_group_flag[grp * 32], epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    while (__hip_atomic_load(&g_fused_group_flag[grp * 32], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
      if (++spins > 100000u) return false;
      __builtin_amdgcn_s_sleep(8);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return true;
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

template <int FMT, bool W_NK>
__global__ __launch_bounds__(256, 1) void linear256_fused_kernel(const GemmArgs g, const uint32_t epoch) {
  __shared__ uint32_t gave_up;
  const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  TileDesc d;  // the stored weight as the forward pass describes it (cols is a multiple of 64 here)
  d.p0 = g.w; d.p1 = g.w_hat; d.p2 = (void*)g.bt; d.p3 = g.scale; d.p4 = nullptr;
  d.b_target = 0.0f; d.b_delta = 1.0f; d.lambda_m = 0.0f;  // g.bt holds b_t itself
  d.ldc = 0; d.first_wg = 0; d.tiles_x_inv = 0;
  d.rows = W_NK ? g.N : g.K; d.cols = W_NK ? g.K : g.N; d.ld = g.ldw;
  d.row0 = g.row0; d.cg0 = g.cg0; d.seed_lo = g.seed_lo; d.seed_hi = g.seed_hi; d.tiles_x = 0;

  // ---- phase 1: sample W once, all wavefronts of the grid ----
  sample_tiles<FMT>(g.step_lo, g.step_hi, d, blockIdx.x * 4 + wave, gridDim.x * 4, lane);
  __syncthreads();
  if (tid == 0) gave_up = grid_arrive_and_wait(epoch) ? 0u : 1u;
  __syncthreads();
  if (gave_up) {  // not every workgroup arrived in time: sample everything here (same bytes)
    sample_tiles<FMT>(g.step_lo, g.step_hi, d, wave, 4, lane);
    __threadfence();
    __syncthreads();
  }

  // ---- phase 2: GEMM tiles on w_hat ----
  const uint32_t total = (g.M / g256::TM) * (g.N / g256::TN);
  for (uint32_t L = blockIdx.x; L < total; L += gridDim.x) {
    gemm256_tile<W_NK>(g, g.w_hat, L);
    __syncthreads();  // the epilogue staging is read before the next tile's loads overwrite it
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

template <int FMT>
static int launch_fused_fmt(const GemmArgs& g, int w_is_nk, uint32_t grid, uint32_t epoch, hipStream_t s) {
  if (w_is_nk) hipLaunchKernelGGL((linear256_fused_kernel<FMT, true>), dim3(grid), dim3(256), 0, s, g, epoch);
  else hipLaunchKernelGGL((linear256_fused_kernel<FMT, false>), dim3(grid), dim3(256), 0, s, g, epoch);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

bool linear256_fused_applicable(const GemmArgs& g) {
  return gemm256_applicable(g) && g.w_hat != nullptr && g.scale != nullptr;
}

int launch_linear256_fused(const GemmArgs& g, int w_is_nk, int fmt, hipStream_t stream) {
  // one workgroup per compute unit: the whole grid is resident, so the arrival counter completes
  const int cus = compute_units();
  if (cus <= 0) return GWS_ERR_LAUNCH;
  static std::atomic<uint32_t> next_epoch{1};
  uint32_t epoch = next_epoch.fetch_add(1);
  if (epoch == 0) epoch = next_epoch.fetch_add(1);
  switch (fmt) {
    case GWS_FMT_BF16: return launch_fused_fmt<0>(g, w_is_nk, (uint32_t)cus, epoch, stream);
    case GWS_FMT_FP8_E4M3: return launch_fused_fmt<1>(g, w_is_nk, (uint32_t)cus, epoch, stream);
    case GWS_FMT_FP6_E3M2: return launch_fused_fmt<2>(g, w_is_nk, (uint32_t)cus, epoch, stream);
    default: return GWS_ERR_FORMAT;
  }
}

}  // namespace gws
