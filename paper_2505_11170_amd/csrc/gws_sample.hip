// GaussWS elementwise kernels: forward (paper Eq. 3 + the cast of Sec. 3.3),
// backward (Eq. 4) and the packed-noise dump (Sec. 3.4), for gfx950.
//
// Work decomposition.  A wavefront owns a 32-row x 64-column tile (two 32x32
// blocks side by side); lane = 8 * r + c loads the 16-byte group of 8 BF16 at
// rows {r, r+8, r+16, r+24}, column group c.  Each load instruction of a wave
// therefore covers 8 rows x 128 contiguous bytes, the four waves of a workgroup
// sit side by side (512 contiguous bytes per row), and the per-block reductions
// (absmax, sum of g.*R) stay inside one wavefront: no LDS, no barrier.
// A workgroup covers one such 32 x 256 tile in the forward pass and up to four
// neighbouring column tiles in the lighter backward pass, where the per-wavefront
// set-up would otherwise show.  Latency is hidden by occupancy: measured on
// MI355X, keeping the next tile's loads in flight inside a wavefront costs more
// in registers than it gains.
// One Philox4x32-10 call yields the 16 bits x 8 elements of one 16-byte group,
// so the noise lives only in registers (2 bytes per parameter of HBM traffic per
// operand, Sec. 3.5; the 0.5 byte per parameter temporary of the paper is gone).
//
// Many tensors per launch: the descriptors travel in the kernel-argument
// segment (no device table, no allocation); a workgroup finds its tensor by a
// scalar scan over the tile prefix.
#include "gws_launch.h"
#include "gws_sample_tile.h"

namespace gws {

// Which tensor, which block-row group and which column strip this workgroup owns, and that
// tensor's descriptor.  Pure scalar work: tile_begin[] ascends, unused entries are
// 0x7FFFFFFF, so (wg - tile_begin[i]) has its top bit clear exactly for the tensors that
// start at or before wg.
// A wavefront lives for one tile, so what it waits for before its first global load counts:
// the prefix table is fetched with four wide scalar loads issued together, the descriptor
// with three, i.e. two scalar-cache round trips in all.  (Left to itself the compiler
// fetches the table in three dependent steps and the descriptor field by field, as each is
// first used: six to nine round trips.)  The empty asm statements pin the loaded values in
// scalar registers at that point, which makes the loads of a batch issue back to back.
typedef uint32_t u32x16s __attribute__((ext_vector_type(16)));
typedef uint32_t u32x8s __attribute__((ext_vector_type(8)));
static_assert(kMaxTensorsPerLaunch == 56 && sizeof(TileDesc) == 96, "locate() is laid out for this table");

__device__ __forceinline__ TileDesc locate(const LaunchArgs& a, uint32_t& byg, uint32_t& bx) {
  const uint32_t wg = blockIdx.x;
  const uint32_t* tb = a.tile_begin;
  u32x16s t0 = *(const u32x16s*)(tb), t1 = *(const u32x16s*)(tb + 16), t2 = *(const u32x16s*)(tb + 32);
  u32x8s t3 = *(const u32x8s*)(tb + 48);
  asm volatile("" : "+s"(t0), "+s"(t1), "+s"(t2), "+s"(t3));
  uint32_t after = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) after += ((wg - t0[i]) >> 31) + ((wg - t1[i]) >> 31) + ((wg - t2[i]) >> 31);
#pragma unroll
  for (int i = 0; i < 8; ++i) after += (wg - t3[i]) >> 31;
  const uint32_t ti = kMaxTensorsPerLaunch - 1 - after;

  const uint32_t* dp = (const uint32_t*)&a.t[ti];
  u32x16s d0 = *(const u32x16s*)(dp);
  u32x8s d1 = *(const u32x8s*)(dp + 16);
  asm volatile("" : "+s"(d0), "+s"(d1));
  uint32_t w[24];
#pragma unroll
  for (int i = 0; i < 16; ++i) w[i] = d0[i];
#pragma unroll
  for (int i = 0; i < 8; ++i) w[16 + i] = d1[i];
  TileDesc d;
  __builtin_memcpy(&d, w, sizeof d);

  // local / tiles_x by the host's reciprocal: the estimate is at most one too small
  const uint32_t local = wg - d.first_wg;
  uint32_t q = __umulhi(local, d.tiles_x_inv);
  uint32_t r = local - q * d.tiles_x;
  if (r >= d.tiles_x) {
    ++q;
    r -= d.tiles_x;
  }
  byg = q;
  bx = r;
  return d;
}

// The tiles of one workgroup: `tiles_per_wg_x` neighbouring column tiles by `tiles_per_wg`
// block rows, column tiles first, so that the workgroups running at any moment cover a
// contiguous stretch of the tensor.  Each wavefront handles its 64-column strip of every
// tile; `body(by, col_base, tile)` is called for strips that exist.  The first tile is
// loaded ahead of the loop, so the common one-tile case stays straight-line code.
template <class F>
__device__ __forceinline__ void walk_tiles(const LaunchArgs& a, const TileDesc& d, uint32_t byg, uint32_t bxg,
                                           F&& body) {
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint32_t r0 = lane >> 3, gcol = (lane & 7) * 8;
  const GWS_GLOBAL uint16_t* __restrict__ src = global_ptr<uint16_t>(d.p0);
  const uint32_t nbr = (d.rows + 31) >> 5, ntx = (d.cols + kTileCols - 1) / kTileCols;
  const uint32_t by0 = byg * a.tiles_per_wg, by_end = min(by0 + a.tiles_per_wg, nbr);
  const uint32_t bx0 = bxg * a.tiles_per_wg_x, bx_end = min(bx0 + a.tiles_per_wg_x, ntx);
  uint32_t by = by0, bx = bx0;
  uint32_t col_base = bx * kTileCols + wave * 64;
  Tile t = load_tile(src, d, by, col_base, col_base + gcol, r0);
  for (;;) {
    if (col_base < d.cols) body(by, col_base, t);
    if (++bx >= bx_end) {
      bx = bx0;
      if (++by >= by_end) break;
    }
    col_base = bx * kTileCols + wave * 64;
    t = load_tile(src, d, by, col_base, col_base + gcol, r0);
  }
}

// MX: write element codes and E8M0 block scales instead of the BF16 container.
// STREAM: non-temporal stores of w_hat (right when it is not read again soon); false keeps w_hat in
// the caches for a GEMM that follows immediately.
// BASIS: the method's bit-built noise, or one of the two comparison bases.
template <int FMT, bool MX = false, bool STREAM = true, int BASIS = kBasisBits>
__global__ __launch_bounds__(kThreads) void sample_fwd_kernel(const LaunchArgs a) {
  uint32_t byg, bxg;
  const TileDesc d = locate(a, byg, bxg);
  const uint32_t lane = threadIdx.x & 63;
  walk_tiles(a, d, byg, bxg, [&](uint32_t by, uint32_t col_base, Tile& t) {
    if (t.full) fwd_tile<FMT, true, STREAM, MX, false, BASIS>(a.step_lo, a.step_hi, d, t, by, col_base, lane);
    else fwd_tile<FMT, false, STREAM, MX, false, BASIS>(a.step_lo, a.step_hi, d, t, by, col_base, lane);
  });
}

template <bool FULL, bool COPY, int BASIS = kBasisBits>
__device__ __forceinline__ void bwd_tile(const LaunchArgs& a, const TileDesc& d, const Tile& t, uint32_t by,
                                         uint32_t col_base, uint32_t lane) {
  const uint32_t row_base = by * 32;
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  const uint32_t col = col_base + gc * 8;
  GWS_GLOBAL uint16_t* __restrict__ dw = global_ptr<uint16_t>(d.p1);
  GWS_GLOBAL float* __restrict__ dbt = global_ptr<float>(d.p2);
  const GWS_GLOBAL float* __restrict__ scale = global_ptr<float>(d.p3);
  const uint32_t cg = d.cg0 + (col >> 3);

  // the block's lane that writes the gradient fetches what it needs first, so the
  // loads are in flight while the noise is regenerated
  const uint32_t nbc = (d.cols + 31) >> 5;
  const uint32_t bcol = (col_base >> 5) + (gc >> 2);
  const bool writer = (FULL || bcol < nbc) && (gc & 3) == 0 && r0 == 0;
  const size_t blk = (size_t)by * nbc + bcol;
  float s32 = 0.0f, bi = 0.0f;
  if (writer) {
    s32 = scale[blk];
    if (d.p4 != nullptr) bi = global_ptr<float>(d.p4)[blk];
  }

  // sum_{b_l}(g .* R), accumulated as sum(g .* 2R) / 2: every product is exact
  // in fp32, the order of the additions is fixed (per lane group by group, two
  // elements per step, then the lane tree), so the result is reproducible.
  float acc = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (!FULL && t.nv[i] == 0) continue;
    const uint32_t row = row_base + r0 + 8 * i;
    if (COPY) {  // dL/dw = dL/dw_hat, bit for bit
      GWS_GLOBAL uint16_t* dst = dw + (size_t)row * d.ld + col;
      if (FULL || t.nv[i] == 8) store16(dst, t.v[i]);
      else store_partial(dst, t.v[i], t.nv[i]);
    }
    const u32x4 gv = (FULL || t.nv[i] == 8) ? t.v[i] : mask_group(t.v[i], t.nv[i]);
    if constexpr (BASIS == kBasisBits) {
      const Noise n = group_noise(cg, d.row0 + row, a.step_lo, a.step_hi, d.seed_lo, d.seed_hi);
      acc = dot_group_2r(gv, n, acc);
    } else {
      const Philox4 x = philox4x32_10(cg, d.row0 + row, a.step_lo, a.step_hi, d.seed_lo, d.seed_hi);
      acc = dot_group_basis<BASIS>(gv, x, acc);
    }
  }
  acc = block_sum_f32(acc) * (BASIS == kBasisBits ? 0.5f : 1.0f);

  if (writer) {
    const float neg_ln2 = __uint_as_float(0xBF317218u);  // -ln 2
    float grad = (neg_ln2 * s32) * acc;                  // dL/db_t, Eq. 4
    if (d.p4 != nullptr) {
      // dL'/db_i, Eq. 11 and Eq. 12: b_t is recomputed exactly as the forward pass formed it,
      // the subgradient of |b_t - b_target| at 0 is taken as 0
      const float btv = __fadd_rn(d.b_target, __fmul_rn(bi, d.b_delta));
      const float sgn = btv > d.b_target ? 1.0f : (btv < d.b_target ? -1.0f : 0.0f);
      grad = d.b_delta * (grad + d.lambda_m * sgn);
    }
    dbt[blk] = grad;
  }
}

template <int BASIS = kBasisBits>
__global__ __launch_bounds__(kThreads) void sample_bwd_kernel(const LaunchArgs a) {
  uint32_t byg, bxg;
  const TileDesc d = locate(a, byg, bxg);
  const uint32_t lane = threadIdx.x & 63;
  const bool copy = d.p1 != nullptr;  // NULL: the pass-through is an alias
  walk_tiles(a, d, byg, bxg, [&](uint32_t by, uint32_t col_base, Tile& t) {
    if (t.full) {
      if (copy) bwd_tile<true, true, BASIS>(a, d, t, by, col_base, lane);
      else bwd_tile<true, false, BASIS>(a, d, t, by, col_base, lane);
    } else {
      if (copy) bwd_tile<false, true, BASIS>(a, d, t, by, col_base, lane);
      else bwd_tile<false, false, BASIS>(a, d, t, by, col_base, lane);
    }
  });
}

// The forward pass for tensors of whole tiles only (rows a multiple of 32, columns of 256): a workgroup walks
// `tiles_per_wg_x` neighbouring column tiles of one block row, straight-line per tile, and keeps the row-only
// share of its Philox calls across them.
template <int FMT, bool MX, bool STREAM>
__global__ __launch_bounds__(kThreads) void sample_fwd_full_kernel(const LaunchArgs a) {
  uint32_t byg, bxg;
  const TileDesc d = locate(a, byg, bxg);
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  const GWS_GLOBAL uint16_t* __restrict__ src = global_ptr<uint16_t>(d.p0);
  const uint32_t ntx = d.cols / kTileCols;
  const uint32_t bx0 = bxg * a.tiles_per_wg_x, bx_end = min(bx0 + a.tiles_per_wg_x, ntx);
  uint32_t rows[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) rows[i] = d.row0 + byg * 32 + r0 + 8 * i;
  const PhiloxRows rp = philox_rows(rows, a.step_lo, d.seed_lo);
  for (uint32_t bx = bx0; bx < bx_end; ++bx) {
    const uint32_t col_base = bx * kTileCols + wave * 64;
    Tile t = load_tile(src, d, byg, col_base, col_base + gc * 8, r0);   // always a whole tile here
    fwd_tile<FMT, true, STREAM, MX>(a.step_lo, a.step_hi, d, t, byg, col_base, lane, 0.0f, &rp);
  }
}

// The backward pass for the shape the method meets in a model: every tensor of the launch has whole tiles only
// (rows a multiple of 32, columns of 256) and dL/dw is an alias (nothing to copy).  Straight-line per tile, and
// the vector ALU work is cut where it can be: the Philox rounds that depend on the row alone are computed once
// per wavefront and reused for every column tile it walks, those that depend on the column group alone once per
// tile (288 vector instructions per tile against about 330 in the kernel for any shape).  The next tile's loads
// are issued after the current tile's arithmetic and complete under the next tile's Philox rounds; issuing them
// a whole tile ahead was measured slower (16 more registers cost a wavefront of occupancy).
__global__ __launch_bounds__(kThreads) void sample_bwd_full_kernel(const LaunchArgs a) {
  uint32_t byg, bxg;
  const TileDesc d = locate(a, byg, bxg);
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  const GWS_GLOBAL uint16_t* __restrict__ src = global_ptr<uint16_t>(d.p0);
  GWS_GLOBAL float* __restrict__ dbt = global_ptr<float>(d.p2);
  const GWS_GLOBAL float* __restrict__ scale = global_ptr<float>(d.p3);
  const uint32_t ntx = d.cols / kTileCols, nbc = d.cols >> 5;
  const uint32_t by = byg;                                                  // one block row per workgroup
  const uint32_t bx0 = bxg * a.tiles_per_wg_x, bx_end = min(bx0 + a.tiles_per_wg_x, ntx);
  const uint32_t row_base = by * 32;
  const bool writer = (gc & 3) == 0 && r0 == 0;

  uint32_t rows[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) rows[i] = d.row0 + row_base + r0 + 8 * i;
  const PhiloxRows rp = philox_rows(rows, a.step_lo, d.seed_lo);

  const GWS_GLOBAL uint16_t* row_ptr = src + (size_t)(row_base + r0) * d.ld + wave * 64 + gc * 8;
  const size_t row_step = (size_t)8 * d.ld;
  u32x4 v[4];
  float s32 = 0.0f, bi = 0.0f;
  auto load4 = [&](uint32_t bx) {
    const GWS_GLOBAL uint16_t* p = row_ptr + (size_t)bx * kTileCols;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = load16(p + i * row_step);
    if (writer) {   // the block's writer lane fetches what it needs with the tile
      const size_t blk = (size_t)by * nbc + ((bx * kTileCols + wave * 64) >> 5) + (gc >> 2);
      s32 = scale[blk];
      if (d.p4 != nullptr) bi = global_ptr<float>(d.p4)[blk];
    }
  };
  load4(bx0);
  for (uint32_t bx = bx0; bx < bx_end; ++bx) {
    const uint32_t col = bx * kTileCols + wave * 64 + gc * 8;
    const PhiloxCols pc = philox_cols(d.cg0 + (col >> 3), a.step_lo, a.step_hi, d.seed_lo, d.seed_hi);
    // sum_{b_l}(g .* R) as sum(g .* 2R) / 2: exact products, fixed order (see bwd_tile)
    float acc = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) acc = dot_group_2r(v[i], noise_planes(philox_row(pc, rp, i, d.seed_lo, d.seed_hi)), acc);
    acc = block_sum_f32(acc) * 0.5f;
    if (writer) {
      const size_t blk = (size_t)by * nbc + (col >> 5);
      const float neg_ln2 = __uint_as_float(0xBF317218u);   // -ln 2
      float grad = (neg_ln2 * s32) * acc;                   // dL/db_t, Eq. 4
      if (d.p4 != nullptr) {                                // dL'/db_i, Eq. 11 and Eq. 12 (as in bwd_tile)
        const float btv = __fadd_rn(d.b_target, __fmul_rn(bi, d.b_delta));
        const float sgn = btv > d.b_target ? 1.0f : (btv < d.b_target ? -1.0f : 0.0f);
        grad = d.b_delta * (grad + d.lambda_m * sgn);
      }
      dbt[blk] = grad;
    }
    if (bx + 1 < bx_end) load4(bx + 1);
  }
}

// The forward kernel's memory traffic without its arithmetic: every tile is loaded and
// stored back unchanged, same workgroup shape, same loads and stores.  What this kernel
// reaches is the ceiling the memory system sets for the access pattern.
__global__ __launch_bounds__(kThreads) void copy_tiles_kernel(const LaunchArgs a) {
  uint32_t byg, bxg;
  const TileDesc d = locate(a, byg, bxg);
  const uint32_t lane = threadIdx.x & 63;
  GWS_GLOBAL uint16_t* __restrict__ dst = global_ptr<uint16_t>(d.p1);
  walk_tiles(a, d, byg, bxg, [&](uint32_t by, uint32_t col_base, Tile& t) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (t.nv[i] == 0) continue;
      GWS_GLOBAL uint16_t* p = dst + (size_t)(by * 32 + (lane >> 3) + 8 * i) * d.ld + col_base + (lane & 7) * 8;
      if (t.nv[i] == 8) store16(p, t.v[i]);
      else store_partial(p, t.v[i], t.nv[i]);
    }
  });
}

// Step one of the forward pass alone: a = max|w| per 32x32 block (exact), written as fp32.
// Reads every element once and writes 4 bytes per block, the traffic profile of the backward
// pass: its rate is the ceiling the memory system sets for a read-only pass of this shape.
__global__ __launch_bounds__(kThreads) void block_absmax_kernel(const LaunchArgs a) {
  uint32_t byg, bxg;
  const TileDesc d = locate(a, byg, bxg);
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  GWS_GLOBAL float* __restrict__ out = global_ptr<float>(d.p3);
  const uint32_t nbc = (d.cols + 31) >> 5;
  walk_tiles(a, d, byg, bxg, [&](uint32_t by, uint32_t col_base, Tile& t) {
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) m = absmax_pk(t.nv[i] < 8 ? mask_group(t.v[i], t.nv[i]) : t.v[i], m);
    m = max(m & 0xFFFFu, m >> 16);
    const uint32_t a16 = block_max_u32(m);
    const uint32_t bcol = (col_base >> 5) + (gc >> 2);
    if (bcol < nbc && (gc & 3) == 0 && r0 == 0) out[(size_t)by * nbc + bcol] = __uint_as_float(a16 << 16);
  });
}

__global__ __launch_bounds__(256) void noise_packed_kernel(uint32_t* __restrict__ out, uint32_t rows,
                                                           uint32_t ngrp, uint32_t row0, uint32_t cg0,
                                                           uint32_t seed_lo, uint32_t seed_hi,
                                                           uint32_t step_lo, uint32_t step_hi) {
  const uint64_t idx = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (uint64_t)rows * ngrp) return;
  const uint32_t row = (uint32_t)(idx / ngrp), cgl = (uint32_t)(idx % ngrp);
  out[idx] = packed_codes(group_noise(cg0 + cgl, row0 + row, step_lo, step_hi, seed_lo, seed_hi));
}

// R of every element under a comparison basis, as BF16 values [rows x 8 ngrp]: one thread per group of 8.
template <int BASIS>
__global__ __launch_bounds__(256) void noise_basis_kernel(u32x4* __restrict__ out, uint32_t rows, uint32_t ngrp,
                                                          uint32_t row0, uint32_t cg0, uint32_t seed_lo, uint32_t seed_hi,
                                                          uint32_t step_lo, uint32_t step_hi) {
  const uint64_t idx = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (uint64_t)rows * ngrp) return;
  const uint32_t row = (uint32_t)(idx / ngrp), cgl = (uint32_t)(idx % ngrp);
  out[idx] = basis_group_bf16<BASIS>(philox4x32_10(cg0 + cgl, row0 + row, step_lo, step_hi, seed_lo, seed_hi));
}

// ---------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------
template <int BASIS>
static int launch_fwd_basis(const LaunchArgs& a, uint32_t n_wg, int fmt, bool keep, hipStream_t stream) {
  if (keep) {
    switch (fmt) {
      case GWS_FMT_BF16: hipLaunchKernelGGL((sample_fwd_kernel<0, false, false, BASIS>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;
      case GWS_FMT_FP8_E4M3: hipLaunchKernelGGL((sample_fwd_kernel<1, false, false, BASIS>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;
      case GWS_FMT_FP6_E3M2: hipLaunchKernelGGL((sample_fwd_kernel<2, false, false, BASIS>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;
      default: return GWS_ERR_FORMAT;
    }
  } else {
    switch (fmt) {
      case GWS_FMT_BF16: hipLaunchKernelGGL((sample_fwd_kernel<0, false, true, BASIS>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;
      case GWS_FMT_FP8_E4M3: hipLaunchKernelGGL((sample_fwd_kernel<1, false, true, BASIS>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;
      case GWS_FMT_FP6_E3M2: hipLaunchKernelGGL((sample_fwd_kernel<2, false, true, BASIS>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;
      default: return GWS_ERR_FORMAT;
    }
  }
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

int launch_sample_fwd_basis(const LaunchArgs& a, uint32_t n_wg, int fmt, bool keep, int basis, hipStream_t stream) {
  if (n_wg == 0) return GWS_OK;
  if (basis == kBasisUniform) return launch_fwd_basis<kBasisUniform>(a, n_wg, fmt, keep, stream);
  if (basis == kBasisBoxMuller) return launch_fwd_basis<kBasisBoxMuller>(a, n_wg, fmt, keep, stream);
  return GWS_ERR_FORMAT;
}

int launch_sample_bwd_basis(const LaunchArgs& a, uint32_t n_wg, int basis, hipStream_t stream) {
  if (n_wg == 0) return GWS_OK;
  if (basis == kBasisUniform) hipLaunchKernelGGL(sample_bwd_kernel<kBasisUniform>, dim3(n_wg), dim3(kThreads), 0, stream, a);
  else if (basis == kBasisBoxMuller) hipLaunchKernelGGL(sample_bwd_kernel<kBasisBoxMuller>, dim3(n_wg), dim3(kThreads), 0, stream, a);
  else return GWS_ERR_FORMAT;
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

int launch_noise_basis(void* out, uint32_t rows, uint32_t ngrp, uint32_t row0, uint32_t cg0, uint64_t seed, uint64_t step,
                       int basis, hipStream_t stream) {
  const uint64_t total = (uint64_t)rows * ngrp;
  if (total == 0) return GWS_OK;
  const uint32_t grid = (uint32_t)((total + 255) / 256);
  const uint32_t slo = (uint32_t)seed, shi = (uint32_t)(seed >> 32), tlo = (uint32_t)step, thi = (uint32_t)(step >> 32);
  if (basis == kBasisUniform)
    hipLaunchKernelGGL(noise_basis_kernel<kBasisUniform>, dim3(grid), dim3(256), 0, stream, (u32x4*)out, rows, ngrp, row0, cg0, slo, shi, tlo, thi);
  else if (basis == kBasisBoxMuller)
    hipLaunchKernelGGL(noise_basis_kernel<kBasisBoxMuller>, dim3(grid), dim3(256), 0, stream, (u32x4*)out, rows, ngrp, row0, cg0, slo, shi, tlo, thi);
  else return GWS_ERR_FORMAT;
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

#define GWS_FWD_CASES(KERNEL)                                                                                             \
  if (mx) {                                                                                                               \
    switch (fmt) {                                                                                                        \
      case GWS_FMT_FP8_E4M3: hipLaunchKernelGGL((KERNEL<1, true, true>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;  \
      case GWS_FMT_FP6_E3M2: hipLaunchKernelGGL((KERNEL<2, true, true>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;  \
      default: return GWS_ERR_FORMAT;                                                                                     \
    }                                                                                                                     \
  } else if (keep) {                                                                                                      \
    switch (fmt) {                                                                                                        \
      case GWS_FMT_BF16: hipLaunchKernelGGL((KERNEL<0, false, false>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;    \
      case GWS_FMT_FP8_E4M3: hipLaunchKernelGGL((KERNEL<1, false, false>), dim3(n_wg), dim3(kThreads), 0, stream, a); break; \
      case GWS_FMT_FP6_E3M2: hipLaunchKernelGGL((KERNEL<2, false, false>), dim3(n_wg), dim3(kThreads), 0, stream, a); break; \
      default: return GWS_ERR_FORMAT;                                                                                     \
    }                                                                                                                     \
  } else {                                                                                                                \
    switch (fmt) {                                                                                                        \
      case GWS_FMT_BF16: hipLaunchKernelGGL((KERNEL<0, false, true>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;     \
      case GWS_FMT_FP8_E4M3: hipLaunchKernelGGL((KERNEL<1, false, true>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;  \
      case GWS_FMT_FP6_E3M2: hipLaunchKernelGGL((KERNEL<2, false, true>), dim3(n_wg), dim3(kThreads), 0, stream, a); break;  \
      default: return GWS_ERR_FORMAT;                                                                                     \
    }                                                                                                                     \
  }

int launch_sample_fwd(const LaunchArgs& a, uint32_t n_wg, int fmt, bool mx, bool keep, int variant, hipStream_t stream) {
  if (n_wg == 0) return GWS_OK;
  if (variant == 1) {
    GWS_FWD_CASES(sample_fwd_full_kernel)
  } else {
    GWS_FWD_CASES(sample_fwd_kernel)
  }
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}
#undef GWS_FWD_CASES

int launch_copy_tiles(const LaunchArgs& a, uint32_t n_wg, hipStream_t stream) {
  if (n_wg == 0) return GWS_OK;
  hipLaunchKernelGGL(copy_tiles_kernel, dim3(n_wg), dim3(kThreads), 0, stream, a);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

int launch_block_absmax(const LaunchArgs& a, uint32_t n_wg, hipStream_t stream) {
  if (n_wg == 0) return GWS_OK;
  hipLaunchKernelGGL(block_absmax_kernel, dim3(n_wg), dim3(kThreads), 0, stream, a);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

int launch_sample_bwd(const LaunchArgs& a, uint32_t n_wg, int variant, hipStream_t stream) {
  if (n_wg == 0) return GWS_OK;
  if (variant == 1) hipLaunchKernelGGL(sample_bwd_full_kernel, dim3(n_wg), dim3(kThreads), 0, stream, a);
  else hipLaunchKernelGGL(sample_bwd_kernel<kBasisBits>, dim3(n_wg), dim3(kThreads), 0, stream, a);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

int launch_noise_packed(uint32_t* out, uint32_t rows, uint32_t ngrp, uint32_t row0, uint32_t cg0,
                        uint64_t seed, uint64_t step, hipStream_t stream) {
  const uint64_t total = (uint64_t)rows * ngrp;
  if (total == 0) return GWS_OK;
  const uint32_t grid = (uint32_t)((total + 255) / 256);
  hipLaunchKernelGGL(noise_packed_kernel, dim3(grid), dim3(256), 0, stream, out, rows, ngrp, row0, cg0,
                     (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)(step >> 32));
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

}  // namespace gws
