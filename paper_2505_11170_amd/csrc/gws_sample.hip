// GaussWS elementwise kernels: forward (paper Eq. 3 + the cast of Sec. 3.3),
// backward (Eq. 4) and the packed-noise dump (Sec. 3.4), for gfx950.
//
// Work decomposition.  A wavefront owns a 32-row x 64-column tile (two 32x32
// blocks side by side); lane = 8 * r + c loads the 16-byte group of 8 BF16 at
// rows {r, r+8, r+16, r+24}, column group c.  Each load instruction of a wave
// therefore covers 8 rows x 128 contiguous bytes, the four waves of a workgroup
// sit side by side (512 contiguous bytes per row), and the per-block reductions
// (absmax, sum of g.*R) stay inside one wavefront: no LDS, no barrier.
// One Philox4x32-10 call yields the 16 bits x 8 elements of one 16-byte group,
// so the noise lives only in registers (2 bytes per parameter of HBM traffic per
// operand, Sec. 3.5; the 0.5 byte per parameter temporary of the paper is gone).
//
// Many tensors per launch: the descriptors travel in the kernel-argument
// segment (no device table, no allocation); a workgroup finds its tensor by a
// scalar scan over the tile prefix.
#include "gws_launch.h"

namespace gws {

// Valid elements of the 16-byte group at (row, col): 8, fewer at a ragged right
// edge, 0 outside.
__device__ __forceinline__ int valid_count(uint32_t row, uint32_t col, uint32_t rows, uint32_t cols) {
  if (row >= rows || col >= cols) return 0;
  const uint32_t left = cols - col;
  return left >= 8 ? 8 : (int)left;
}

__device__ __forceinline__ void locate(const LaunchArgs& a, int& ti, uint32_t& by, uint32_t& bx) {
  const uint32_t wg = blockIdx.x;
  ti = 0;
  for (int i = 1; i < (int)a.n; ++i)
    if (a.t[i].tile_begin <= wg) ti = i;
  const uint32_t local = wg - a.t[ti].tile_begin;
  by = local / a.t[ti].tiles_x;
  bx = local - by * a.t[ti].tiles_x;
}

template <int FMT>
__global__ __launch_bounds__(kThreads) void sample_fwd_kernel(const LaunchArgs a) {
  int ti;
  uint32_t by, bx;
  locate(a, ti, by, bx);
  const TileDesc& d = a.t[ti];
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint32_t col_base = bx * kTileCols + wave * 64;
  if (col_base >= d.cols) return;  // whole wavefront past the right edge
  const uint32_t row_base = by * 32;
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  const uint32_t col = col_base + gc * 8;
  const uint16_t* __restrict__ w = (const uint16_t*)d.p0;
  uint16_t* __restrict__ w_hat = (uint16_t*)d.p1;
  const float* __restrict__ bt = (const float*)d.p2;
  float* __restrict__ scale = (float*)d.p3;
  const bool full = (row_base + 32 <= d.rows) && (col_base + 64 <= d.cols);

  // ---- load the tile (a 16-byte load never leaves its row: ld % 8 == 0) ----
  uint4 v[4];
  int nv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t row = row_base + r0 + 8 * i;
    nv[i] = full ? 8 : valid_count(row, col, d.rows, d.cols);
    v[i] = make_uint4(0, 0, 0, 0);
    if (nv[i] > 0) v[i] = *(const uint4*)(w + (size_t)row * d.ld + col);
    if (nv[i] > 0 && nv[i] < 8) {  // ragged right edge: elements past cols do not exist
      uint32_t e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k >= nv[i]) e[k >> 1] &= (k & 1) ? 0x0000FFFFu : 0xFFFF0000u;
      v[i] = make_uint4(e[0], e[1], e[2], e[3]);
    }
  }

  // ---- a = max_{b_l}|w| on the magnitude bits (exact) ----
  uint32_t m = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      m = max(m, e[k] & 0x7FFFu);
      m = max(m, (e[k] >> 16) & 0x7FFFu);
    }
  }
  const uint32_t a16 = block_max_u32(m);

  // ---- per-block scale ----
  const uint32_t nbc = (d.cols + 31) >> 5;
  const uint32_t bcol = (col_base >> 5) + (gc >> 2);
  const bool block_exists = bcol < nbc;
  const float btv = block_exists ? bt[(size_t)by * nbc + bcol] : 0.0f;
  BlockScale b = block_scale(a16, btv);
  if (FMT == 1) cast_constants<8, -6>(a16, b);
  if (FMT == 2) cast_constants<4, -2>(a16, b);
  if (block_exists && (gc & 3) == 0 && r0 == 0) scale[(size_t)by * nbc + bcol] = b.s32;

  // ---- noise, add, round, cast, store ----
  const uint32_t cg = d.cg0 + (col >> 3);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (nv[i] == 0) continue;
    const uint32_t row = row_base + r0 + 8 * i;
    const uint32_t codes = group_codes(cg, d.row0 + row, a.step_lo, a.step_hi, d.seed_lo, d.seed_hi);
    const uint32_t e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t lo = sample_element<FMT>(__uint_as_float(e[k] << 16), (codes >> (8 * k)) & 0xFu, b);
      const uint32_t hi =
          sample_element<FMT>(__uint_as_float(e[k] & 0xFFFF0000u), (codes >> (8 * k + 4)) & 0xFu, b);
      o[k] = lo | (hi << 16);
    }
    uint16_t* dst = w_hat + (size_t)row * d.ld + col;
    if (nv[i] == 8) {
      *(uint4*)dst = make_uint4(o[0], o[1], o[2], o[3]);
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k < nv[i]) dst[k] = (uint16_t)(o[k >> 1] >> ((k & 1) * 16));
    }
  }
}

__global__ __launch_bounds__(kThreads) void sample_bwd_kernel(const LaunchArgs a) {
  int ti;
  uint32_t by, bx;
  locate(a, ti, by, bx);
  const TileDesc& d = a.t[ti];
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint32_t col_base = bx * kTileCols + wave * 64;
  if (col_base >= d.cols) return;
  const uint32_t row_base = by * 32;
  const uint32_t gc = lane & 7, r0 = lane >> 3;
  const uint32_t col = col_base + gc * 8;
  const uint16_t* __restrict__ g = (const uint16_t*)d.p0;
  uint16_t* __restrict__ dw = (uint16_t*)d.p1;  // NULL: pass-through is an alias
  float* __restrict__ dbt = (float*)d.p2;
  const float* __restrict__ scale = (const float*)d.p3;
  const bool full = (row_base + 32 <= d.rows) && (col_base + 64 <= d.cols);
  const uint32_t cg = d.cg0 + (col >> 3);

  uint4 v[4];
  int nv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t row = row_base + r0 + 8 * i;
    nv[i] = full ? 8 : valid_count(row, col, d.rows, d.cols);
    v[i] = make_uint4(0, 0, 0, 0);
    if (nv[i] > 0) v[i] = *(const uint4*)(g + (size_t)row * d.ld + col);
  }

  // sum_{b_l}(g .* R): every product is exact in fp32 (R in {0, +-1, +-2}); the
  // order of the additions is fixed (i, then k, then the lane tree), so the
  // result is reproducible bit for bit.
  float acc = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (nv[i] == 0) continue;
    const uint32_t row = row_base + r0 + 8 * i;
    const uint32_t codes = group_codes(cg, d.row0 + row, a.step_lo, a.step_hi, d.seed_lo, d.seed_hi);
    const uint32_t e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const uint32_t code = (codes >> (4 * k)) & 0xFu;
      const float mag = (float)(code & 3u);
      const float r = __uint_as_float(__float_as_uint(mag) | ((code & 8u) << 28));
      const float gv = __uint_as_float((k & 1) ? (e[k >> 1] & 0xFFFF0000u) : (e[k >> 1] << 16));
      if (k < nv[i]) acc += gv * r;
    }
    if (dw != nullptr) {  // dL/dw = dL/dw_hat, bit for bit
      uint16_t* dst = dw + (size_t)row * d.ld + col;
      if (nv[i] == 8) {
        *(uint4*)dst = v[i];
      } else {
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (k < nv[i]) dst[k] = (uint16_t)(e[k >> 1] >> ((k & 1) * 16));
      }
    }
  }
  acc = block_sum_f32(acc);

  const uint32_t nbc = (d.cols + 31) >> 5;
  const uint32_t bcol = (col_base >> 5) + (gc >> 2);
  if (bcol < nbc && (gc & 3) == 0 && r0 == 0) {
    const float s32 = scale[(size_t)by * nbc + bcol];
    const float neg_ln2 = __uint_as_float(0xBF317218u);  // -ln 2
    dbt[(size_t)by * nbc + bcol] = (neg_ln2 * s32) * acc;
  }
}

__global__ __launch_bounds__(256) void noise_packed_kernel(uint32_t* __restrict__ out, uint32_t rows,
                                                           uint32_t ngrp, uint32_t row0, uint32_t cg0,
                                                           uint32_t seed_lo, uint32_t seed_hi,
                                                           uint32_t step_lo, uint32_t step_hi) {
  const uint64_t idx = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (uint64_t)rows * ngrp) return;
  const uint32_t row = (uint32_t)(idx / ngrp), cgl = (uint32_t)(idx % ngrp);
  out[idx] = group_codes(cg0 + cgl, row0 + row, step_lo, step_hi, seed_lo, seed_hi);
}

// ---------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------
int launch_sample_fwd(const LaunchArgs& a, uint32_t n_tiles, int fmt, hipStream_t stream) {
  if (n_tiles == 0) return GWS_OK;
  switch (fmt) {
    case GWS_FMT_BF16: hipLaunchKernelGGL(sample_fwd_kernel<0>, dim3(n_tiles), dim3(kThreads), 0, stream, a); break;
    case GWS_FMT_FP8_E4M3: hipLaunchKernelGGL(sample_fwd_kernel<1>, dim3(n_tiles), dim3(kThreads), 0, stream, a); break;
    case GWS_FMT_FP6_E3M2: hipLaunchKernelGGL(sample_fwd_kernel<2>, dim3(n_tiles), dim3(kThreads), 0, stream, a); break;
    default: return GWS_ERR_FORMAT;
  }
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

int launch_sample_bwd(const LaunchArgs& a, uint32_t n_tiles, hipStream_t stream) {
  if (n_tiles == 0) return GWS_OK;
  hipLaunchKernelGGL(sample_bwd_kernel, dim3(n_tiles), dim3(kThreads), 0, stream, a);
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
