// Launch descriptors shared by the host API and the kernels (internal to csrc/).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gws.h"
#include "gws_device.h"

namespace gws {

constexpr int kThreads = 256;       // 4 wavefronts per workgroup
constexpr int kTileCols = 256;      // a workgroup covers 32 rows x 256 columns
constexpr int kMaxTensorsPerLaunch = 56;

// One tensor as a kernel sees it.  p0..p3 are, for the forward pass,
// (w, w_hat, bt-or-b_i, scale) and, for the backward pass, (g, dw-or-NULL,
// dbt-or-db_i, scale); p4 is the backward pass's b_i (NULL: the gradient asked
// for is dL/db_t itself).  The forward pass with MX output carries the element
// codes in p1 (row stride ldc bytes) and the E8M0 block scales in p4.
// The bitwidth a block uses is b_t = b_target + v * b_delta (paper Eq. 11) with v
// the value read through p2; a plain b_t input is the case b_target = 0,
// b_delta = 1, which leaves every finite value as it is.
struct TileDesc {
  const void* p0;
  void* p1;
  void* p2;
  void* p3;
  void* p4;
  uint32_t rows, cols, ld;
  uint32_t row0, cg0;          // shard origin: row offset, column-group (col0 / 8) offset
  uint32_t seed_lo, seed_hi;
  uint32_t tiles_x;            // workgroups per row of workgroups = ceil(ceil(cols / 256) / tiles_per_wg_x)
  float b_target, b_delta;     // Eq. 11: b_delta = b_init - b_target
  float lambda_m;              // Eq. 12: lambda / (blocks of the layer); backward only
  uint32_t ldc;                // MX output: bytes per row of element codes
  uint32_t first_wg;           // this tensor's first workgroup within the launch (= its tile_begin entry)
  uint32_t tiles_x_inv;        // min(floor(2^32 / tiles_x), 2^32 - 1): division by multiplication in locate()
};
static_assert(sizeof(TileDesc) == 96, "descriptor layout");

// Passed by value: lives in the kernel-argument segment (about 5.5 KiB; the segment
// of a gfx950 code object is not limited to 4 KiB).
struct LaunchArgs {
  // First workgroup of every tensor within the launch; entries past n hold 0x7FFFFFFF.
  // Kept apart from the descriptors so a wavefront reads the whole prefix with a few
  // wide scalar loads instead of one dependent load per tensor.
  uint32_t tile_begin[kMaxTensorsPerLaunch];
  TileDesc t[kMaxTensorsPerLaunch];
  uint32_t n;
  uint32_t step_lo, step_hi;
  uint32_t tiles_per_wg;       // consecutive block rows one workgroup covers (>= 1)
  uint32_t tiles_per_wg_x;     // neighbouring 256-column tiles one workgroup covers (>= 1)
};
static_assert(sizeof(LaunchArgs) <= 6144, "kernel arguments: keep within the size verified on the device");

// variant: 0 = any shape (sample_fwd_kernel); 1 = whole tiles only (sample_fwd_full_kernel)
int launch_sample_fwd(const LaunchArgs& a, uint32_t n_wg, int fmt, bool mx, bool keep, int variant, hipStream_t stream);
// variant: 0 = any shape (sample_bwd_kernel); 1 = whole tiles and aliased dL/dw only (sample_bwd_full_kernel)
int launch_sample_bwd(const LaunchArgs& a, uint32_t n_wg, int variant, hipStream_t stream);
// the same two passes with R drawn from a comparison basis (kBasisUniform, kBasisBoxMuller)
int launch_sample_fwd_basis(const LaunchArgs& a, uint32_t n_wg, int fmt, bool keep, int basis, hipStream_t stream);
int launch_sample_bwd_basis(const LaunchArgs& a, uint32_t n_wg, int basis, hipStream_t stream);
int launch_noise_basis(void* out, uint32_t rows, uint32_t ngrp, uint32_t row0, uint32_t cg0, uint64_t seed, uint64_t step,
                       int basis, hipStream_t stream);
int launch_copy_tiles(const LaunchArgs& a, uint32_t n_wg, hipStream_t stream);
int launch_block_absmax(const LaunchArgs& a, uint32_t n_wg, hipStream_t stream);
int launch_noise_packed(uint32_t* out, uint32_t rows, uint32_t ngrp, uint32_t row0, uint32_t cg0,
                        uint64_t seed, uint64_t step, hipStream_t stream);

// GEMM launchers (gws_linear.hip)
struct GemmArgs {
  const uint16_t* x;   // [M x K], ldx
  const uint16_t* w;   // [K x N] or [N x K], ldw
  uint16_t* y;         // [M x N], ldy
  uint32_t M, N, K;
  uint32_t ldx, ldw, ldy;
  // sampling (fused variant only)
  const float* bt;
  float* scale;        // may be NULL
  uint16_t* w_hat;     // may be NULL
  uint32_t row0, cg0, seed_lo, seed_hi, step_lo, step_hi;
  float* dbt;          // weight-gradient GEMM only: dL/db_t per block (with scale as input)
};
// fused: 0 = plain GEMM on g.w; kFusedInOperand = sampling in the weight operand load of every tile
constexpr int kFusedInOperand = 2;
int launch_gemm(const GemmArgs& g, int w_is_nk, int fused, int fmt, hipStream_t stream);
bool gemm256_applicable(const GemmArgs& g);
int launch_gemm256(const GemmArgs& g, int w_is_nk, hipStream_t stream);
// Weights whose forward sampling rides in a GEMM's launch: descriptors as the forward pass fills them, with
// first_wg = the weight's first 32 x 256 tile in the riders' numbering (rider 1); begin[j] = that number again for
// j < n and the total for every j >= n (so that a search over begin[1..] needs no n).
constexpr int kMaxRide = 4;
struct RideList {
  TileDesc d[kMaxRide];
  uint32_t begin[kMaxRide + 1];
  uint32_t n;
};
// the 256-tile GEMM (none if g.M == 0) followed, in the same grid, by `extra` workgroups that sample the weights of
// `r` as the forward pass does; rider: 0 = sample_tiles on r.d[0] alone (rows a multiple of 32, columns of 64),
// 1 = ride_tiles (every weight: rows a multiple of 32, columns of 256)
int launch_gemm256_ride(const GemmArgs& g, int w_is_nk, const RideList& r, int fmt, uint64_t step, uint32_t extra,
                        int rider, hipStream_t stream);
int compute_units();   // of the current device; 0 if the query fails
// Weight-gradient GEMM (gws_gemm256_tn.hip): y[M x N] = x^T * w with x [K x M], w [K x N]
// row-major (K = the contraction length); with_dbt adds Eq. 4's block reduction on y.
bool gemm256_tn_applicable(const GemmArgs& g);
int launch_gemm256_tn(const GemmArgs& g, bool with_dbt, hipStream_t stream);
// the same result with the contraction of every tile split over `parts` (2 .. K / 64) workgroups: fp32 partial tiles in
// `ws` (gemm256_tn_split_bytes, 16-byte aligned), added in a fixed order by a second kernel
size_t gemm256_tn_split_bytes(const GemmArgs& g, uint32_t parts);
int launch_gemm256_tn_split(const GemmArgs& g, bool with_dbt, float* ws, uint32_t parts, hipStream_t stream);

}  // namespace gws
