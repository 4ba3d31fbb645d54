// C ABI of libgws: argument validation and launch planning.  Declarations and
// the meaning of every argument are in include/gws.h.
#include <string.h>

#include <atomic>

#include "gws_bench.h"
#include "gws_launch.h"

// Staging buffer of gws_linear_fwd_static: device memory that belongs to the loaded code object, one copy
// per GPU.  Host code never uses this name as an address: it asks the runtime for the device address
// (scratch_of_current_device) and passes that to the kernels like any other buffer.
static __device__ __align__(256) unsigned char scratch[GWS_STATIC_SCRATCH_BYTES];

namespace {

using namespace gws;

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_addr[kMaxDevices];   // device address of `scratch` on each GPU, once looked up

// The address of `scratch` on the current device (looked up once per device, with that device current).
int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GWS_ERR_LAUNCH;
  void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return GWS_ERR_LAUNCH;
    g_scratch_addr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return GWS_OK;
}

inline bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Shape rules common to forward and backward.
int check_shape(const gws_tensor& t) {
  if (t.rows < 0 || t.cols < 0 || t.ld < 0) return GWS_ERR_SHAPE;
  if (t.rows >= (int64_t)1 << 31 || t.cols >= (int64_t)1 << 31 || t.ld >= (int64_t)1 << 31) return GWS_ERR_SHAPE;
  if (t.rows == 0 || t.cols == 0) return GWS_OK;
  if (t.ld < t.cols || (t.ld & 7) != 0) return GWS_ERR_SHAPE;
  if (t.row0 < 0 || t.col0 < 0 || (t.row0 & 31) != 0 || (t.col0 & 31) != 0) return GWS_ERR_SHAPE;
  if (t.row0 + t.rows > (int64_t)0xFFFFFFFFll || (t.col0 + t.cols) / 8 > (int64_t)0xFFFFFFFFll) return GWS_ERR_SHAPE;
  return GWS_OK;
}

inline bool overlap(const void* a, const void* b, size_t bytes) {
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + bytes && y < x + bytes;
}

int check_fwd(const gws_tensor& t) {
  int rc = check_shape(t);
  if (rc != GWS_OK || t.rows == 0 || t.cols == 0) return rc;
  if (!t.w || !t.w_hat || !t.bt || !t.scale) return GWS_ERR_NULL;
  if (!aligned(t.w, 16) || !aligned(t.w_hat, 16) || !aligned(t.bt, 4) || !aligned(t.scale, 4)) return GWS_ERR_ALIGN;
  if (overlap(t.w, t.w_hat, (size_t)t.rows * t.ld * 2)) return GWS_ERR_ALIAS;
  return GWS_OK;
}

inline bool overlap2(const void* a, size_t abytes, const void* b, size_t bbytes) {
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + bbytes && y < x + abytes;
}

int check_fwd_mx(const gws_tensor& t, const gws_mx_out& o, int fmt) {
  int rc = check_shape(t);
  if (rc != GWS_OK || t.rows == 0 || t.cols == 0) return rc;
  if (!t.w || !t.bt || !t.scale || !o.codes || !o.xscale) return GWS_ERR_NULL;
  const bool fp8 = fmt == GWS_FMT_FP8_E4M3;
  const int64_t row_bytes = fp8 ? t.cols : (t.cols * 6 + 7) / 8;
  if (o.ldc < row_bytes || o.ldc >= (int64_t)1 << 31 || (o.ldc & (fp8 ? 7 : 1)) != 0) return GWS_ERR_SHAPE;
  if (!aligned(t.w, 16) || !aligned(t.bt, 4) || !aligned(t.scale, 4) || !aligned(o.codes, fp8 ? 8 : 2)) return GWS_ERR_ALIGN;
  if (overlap2(t.w, (size_t)t.rows * t.ld * 2, o.codes, (size_t)t.rows * o.ldc)) return GWS_ERR_ALIAS;
  return GWS_OK;
}

int check_bwd(const gws_tensor& t) {
  int rc = check_shape(t);
  if (rc != GWS_OK || t.rows == 0 || t.cols == 0) return rc;
  if (!t.g || !t.dbt || !t.scale) return GWS_ERR_NULL;
  if (!aligned(t.g, 16) || !aligned(t.dw, 16) || !aligned(t.dbt, 4) || !aligned(t.scale, 4)) return GWS_ERR_ALIGN;
  if (t.dw && t.dw != t.g && overlap(t.g, t.dw, (size_t)t.rows * t.ld * 2)) return GWS_ERR_ALIAS;
  return GWS_OK;
}

void fill_common(TileDesc& d, const gws_tensor& t, uint32_t per_x) {
  d.rows = (uint32_t)t.rows;
  d.cols = (uint32_t)t.cols;
  d.ld = (uint32_t)t.ld;
  d.row0 = (uint32_t)t.row0;
  d.cg0 = (uint32_t)(t.col0 / 8);
  d.seed_lo = (uint32_t)t.seed;
  d.seed_hi = (uint32_t)(t.seed >> 32);
  d.tiles_x = (uint32_t)(((t.cols + kTileCols - 1) / kTileCols + per_x - 1) / per_x);
  const uint64_t inv = ((uint64_t)1 << 32) / d.tiles_x;
  d.tiles_x_inv = inv > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)inv;
}

// Workgroups a tensor needs when each covers `per_wg` block rows by `per_x` 256-column tiles.
inline uint64_t wg_count(const gws_tensor& t, uint32_t per_wg, uint32_t per_x) {
  const uint64_t nbr = (uint64_t)((t.rows + 31) / 32);
  const uint64_t ntx = (uint64_t)((t.cols + kTileCols - 1) / kTileCols);
  return ((nbr + per_wg - 1) / per_wg) * ((ntx + per_x - 1) / per_x);
}

constexpr int kCopyOnly = -1;    // run_batched "format": the forward launch shape, copy kernel
constexpr int kAbsmaxOnly = -2;  // the backward launch shape, block-maximum kernel (descriptor: w, scale)

// Pack descriptors into as few launches as the kernel-argument segment and the
// 2^31 grid limit allow.  `fwd` selects which pointers a descriptor carries.
// `bw` (one per tensor) switches on the parametrised bitwidth of Eq. 11 / Eq. 12.
// `mx` (one per tensor, forward only) switches the output to MX element codes and block scales.
// Launch-shape choices of a sampling pass; the defaults (-1, 0) let run_batched decide.
struct Tuning {
  int variant = -1;   // launch_sample_fwd's / launch_sample_bwd's variant; above 0 only where every tensor qualifies
  int per_x = 0;      // column tiles per workgroup
};

// `basis` other than kBasisBits runs the sampling passes on a comparison noise basis (no bw, no mx then).
int run_batched(const gws_tensor* t, int n, const gws_bitwidth* bw, const gws_mx_out* mx, bool fwd, int fmt,
                uint64_t step, hipStream_t stream, bool keep = false, int basis = kBasisBits,
                Tuning tune = Tuning()) {
  // Tiles per workgroup.  Forward: one (most workgroups; measured best: 2 costs 1-10 %, 4 costs 6-10 %).
  // Backward does less per tile, so the per-wavefront set-up shows, and its Philox rounds that depend on
  // the row alone are reused across column tiles: a workgroup takes up to four neighbouring column tiles
  // while at least ~3000 workgroups (12 per compute unit) remain (measured: 3 best on the 85 M parameters
  // of GPT2-124M, 4 on the 1B model; 6 and more lose).  Neighbouring column tiles, not rows: the
  // workgroups in flight then still cover a contiguous stretch of memory, which the memory system rewards.
  uint64_t total = 0;
  for (int i = 0; i < n; ++i)
    if (t[i].rows > 0 && t[i].cols > 0) total += wg_count(t[i], 1, 1);
  uint32_t per_wg = 1, per_x = 1;
  if (!fwd) {
    while (per_x < 4 && total / (per_x + 1) >= 3000) ++per_x;
  }
  if (tune.per_x > 0) per_x = (uint32_t)tune.per_x;
  // Forward stores: a call that writes little (one weight, a few layers) is usually followed by its
  // consumer, and the whole of w_hat fits in the last-level cache, so it is written with ordinary
  // stores; a call over a model's worth of weights streams past the caches (non-temporal stores).
  // A workgroup tile is 32 x 256 elements = 16 KiB of w_hat.
  if (fwd && total * (16u << 10) <= (32u << 20)) keep = true;

  LaunchArgs a;
  memset(&a, 0, sizeof a);
  a.step_lo = (uint32_t)step;
  a.step_hi = (uint32_t)(step >> 32);
  a.tiles_per_wg = per_wg;
  a.tiles_per_wg_x = per_x;
  for (int i = 0; i < kMaxTensorsPerLaunch; ++i) a.tile_begin[i] = 0x7FFFFFFFu;
  uint64_t wgs = 0;
  bool whole_tiles = true;   // every tensor of the pending launch: rows % 32 == 0, cols % 256 == 0, nothing to copy
  auto flush = [&]() -> int {
    if (a.n == 0) return GWS_OK;
    const int variant = !whole_tiles ? 0 : tune.variant >= 0 ? tune.variant : 1;
    int rc = (!fwd && fmt == kAbsmaxOnly) ? launch_block_absmax(a, (uint32_t)wgs, stream)
             : (!fwd && basis != kBasisBits) ? launch_sample_bwd_basis(a, (uint32_t)wgs, basis, stream)
             : !fwd ? launch_sample_bwd(a, (uint32_t)wgs, variant, stream)
             : fmt == kCopyOnly ? launch_copy_tiles(a, (uint32_t)wgs, stream)
             : basis != kBasisBits ? launch_sample_fwd_basis(a, (uint32_t)wgs, fmt, keep, basis, stream)
                                   : launch_sample_fwd(a, (uint32_t)wgs, fmt, mx != nullptr, keep, variant, stream);
    a.n = 0;
    wgs = 0;
    whole_tiles = true;
    for (int i = 0; i < kMaxTensorsPerLaunch; ++i) a.tile_begin[i] = 0x7FFFFFFFu;
    return rc;
  };
  for (int i = 0; i < n; ++i) {
    if (t[i].rows == 0 || t[i].cols == 0) continue;
    const uint64_t wc = wg_count(t[i], per_wg, per_x);
    if (wc >= 0x7FFFFFF0ull) return GWS_ERR_SHAPE;
    if (a.n == (uint32_t)kMaxTensorsPerLaunch || wgs + wc >= 0x7FFFFFF0ull) {
      int rc = flush();
      if (rc != GWS_OK) return rc;
    }
    a.tile_begin[a.n] = (uint32_t)wgs;
    TileDesc& d = a.t[a.n++];
    d.first_wg = (uint32_t)wgs;
    if (fwd) {
      d.p0 = t[i].w; d.p1 = t[i].w_hat; d.p2 = (void*)t[i].bt; d.p3 = t[i].scale;
      if ((t[i].rows & 31) != 0 || (t[i].cols & (kTileCols - 1)) != 0) whole_tiles = false;
    } else if (fmt == kAbsmaxOnly) {
      d.p0 = t[i].w; d.p1 = nullptr; d.p2 = nullptr; d.p3 = t[i].scale;
    } else {
      d.p0 = t[i].g; d.p1 = (t[i].dw == t[i].g) ? nullptr : t[i].dw; d.p2 = t[i].dbt; d.p3 = t[i].scale;
      if (d.p1 != nullptr || (t[i].rows & 31) != 0 || (t[i].cols & (kTileCols - 1)) != 0) whole_tiles = false;
    }
    fill_common(d, t[i], per_x);
    d.p4 = nullptr;
    d.b_target = 0.0f;
    d.b_delta = 1.0f;
    d.lambda_m = 0.0f;
    d.ldc = 0;
    if (mx) {
      d.p1 = mx[i].codes;
      d.p4 = mx[i].xscale;
      d.ldc = (uint32_t)mx[i].ldc;
    }
    if (bw) {
      d.b_target = bw[i].b_target;
      d.b_delta = bw[i].b_init - bw[i].b_target;
      if (!fwd) {
        const int64_t own = ((t[i].rows + 31) / 32) * ((t[i].cols + 31) / 32);
        const int64_t m = bw[i].layer_blocks > 0 ? bw[i].layer_blocks : own;
        d.p4 = (void*)t[i].bt;
        d.lambda_m = bw[i].lambda / (float)m;
      }
    }
    wgs += wc;
  }
  return flush();
}

// Argument rules shared by the forms of the sampled-weight linear (w is not NULL).  Returns GWS_OK
// also for an empty product (M == 0 or N == 0), which the caller skips.
int check_linear(const void* x, int64_t M, int64_t K, int64_t ldx, const gws_tensor* w, int w_is_nk, const void* y,
                 int64_t ldy) {
  int rc = check_shape(*w);
  if (rc != GWS_OK) return rc;
  const int64_t Kw = w_is_nk ? w->cols : w->rows, N = w_is_nk ? w->rows : w->cols;
  if (M < 0 || K < 0 || K != Kw || M >= (int64_t)1 << 31) return GWS_ERR_SHAPE;
  if (M == 0 || N == 0) return GWS_OK;
  if ((K & 31) != 0 || (N & 31) != 0 || K == 0) return GWS_ERR_SHAPE;
  if (ldx < K || ldy < N || (ldx & 7) != 0 || (ldy & 7) != 0 || ldx >= (int64_t)1 << 31 || ldy >= (int64_t)1 << 31) return GWS_ERR_SHAPE;
  if (!x || !y || !w->w || !w->bt) return GWS_ERR_NULL;
  if (!aligned(x, 16) || !aligned(y, 16) || !aligned(w->w, 16) || !aligned(w->bt, 4)) return GWS_ERR_ALIGN;
  return GWS_OK;
}

GemmArgs linear_args(const void* x, int64_t M, int64_t K, int64_t ldx, const gws_tensor* w, int w_is_nk, uint64_t step,
                     void* y, int64_t ldy) {
  GemmArgs g;
  memset(&g, 0, sizeof g);
  g.x = (const uint16_t*)x; g.w = (const uint16_t*)w->w; g.y = (uint16_t*)y;
  g.M = (uint32_t)M; g.N = (uint32_t)(w_is_nk ? w->rows : w->cols); g.K = (uint32_t)K;
  g.ldx = (uint32_t)ldx; g.ldw = (uint32_t)w->ld; g.ldy = (uint32_t)ldy;
  g.bt = w->bt;
  g.row0 = (uint32_t)w->row0; g.cg0 = (uint32_t)(w->col0 / 8);
  g.seed_lo = (uint32_t)w->seed; g.seed_hi = (uint32_t)(w->seed >> 32);
  g.step_lo = (uint32_t)step; g.step_hi = (uint32_t)(step >> 32);
  return g;
}

// Bytes of the staged w_hat of a weight, rounded up so that the block scales behind it stay aligned.
inline size_t staged_bytes(const gws_tensor& w) { return (((size_t)w.rows * (size_t)w.ld * 2) + 255) & ~(size_t)255; }

// The sampled-weight linear with w_hat and scale staged in `staging` (device, 256-byte aligned, at least
// gws_linear_fwd_workspace_bytes(w)): the sampling kernel writes them there, the plain GEMM reads w_hat.
// Arguments already checked.
int linear_staged(const void* x, int64_t M, int64_t K, int64_t ldx, const gws_tensor* w, int w_is_nk, int fmt,
                  uint64_t step, void* y, int64_t ldy, void* staging, hipStream_t stream) {
  gws_tensor t = *w;
  t.w_hat = staging;
  t.scale = (float*)((char*)staging + staged_bytes(*w));
  const size_t w_bytes = (size_t)w->rows * w->ld * 2, need = staged_bytes(*w) + (size_t)((w->rows + 31) / 32) * ((w->cols + 31) / 32) * 4;
  if (overlap2(staging, need, w->w, w_bytes) || overlap2(staging, need, x, (size_t)M * ldx * 2) ||
      overlap2(staging, need, y, (size_t)M * ldy * 2)) return GWS_ERR_ALIAS;
  int rc = run_batched(&t, 1, nullptr, nullptr, true, fmt, step, stream, /*keep=*/true);
  if (rc != GWS_OK) return rc;
  GemmArgs g = linear_args(x, M, K, ldx, w, w_is_nk, step, y, ldy);
  g.w = (const uint16_t*)staging;
  return launch_gemm(g, w_is_nk, 0, GWS_FMT_BF16, stream);
}

}  // namespace

extern "C" {

int gws_sample_fwd(const gws_tensor* t, int n, int fmt, uint64_t step, void* stream) {
  if (n < 0) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t) return GWS_ERR_NULL;
  if (fmt != GWS_FMT_BF16 && fmt != GWS_FMT_FP8_E4M3 && fmt != GWS_FMT_FP6_E3M2) return GWS_ERR_FORMAT;
  for (int i = 0; i < n; ++i) {
    int rc = check_fwd(t[i]);
    if (rc != GWS_OK) return rc;
  }
  return run_batched(t, n, nullptr, nullptr, true, fmt, step, (hipStream_t)stream);
}

int gws_sample_bwd(const gws_tensor* t, int n, uint64_t step, void* stream) {
  if (n < 0) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t) return GWS_ERR_NULL;
  for (int i = 0; i < n; ++i) {
    int rc = check_bwd(t[i]);
    if (rc != GWS_OK) return rc;
  }
  return run_batched(t, n, nullptr, nullptr, false, 0, step, (hipStream_t)stream);
}

int gws_sample_fwd_basis(const gws_tensor* t, int n, int basis, int fmt, uint64_t step, void* stream) {
  if (basis == GWS_BASIS_BITS) return gws_sample_fwd(t, n, fmt, step, stream);
  if (basis != GWS_BASIS_UNIFORM_BF16 && basis != GWS_BASIS_BOX_MULLER) return GWS_ERR_FORMAT;
  if (n < 0) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t) return GWS_ERR_NULL;
  if (fmt != GWS_FMT_BF16 && fmt != GWS_FMT_FP8_E4M3 && fmt != GWS_FMT_FP6_E3M2) return GWS_ERR_FORMAT;
  for (int i = 0; i < n; ++i) {
    int rc = check_fwd(t[i]);
    if (rc != GWS_OK) return rc;
  }
  return run_batched(t, n, nullptr, nullptr, true, fmt, step, (hipStream_t)stream, false, basis);
}

int gws_sample_bwd_basis(const gws_tensor* t, int n, int basis, uint64_t step, void* stream) {
  if (basis == GWS_BASIS_BITS) return gws_sample_bwd(t, n, step, stream);
  if (basis != GWS_BASIS_UNIFORM_BF16 && basis != GWS_BASIS_BOX_MULLER) return GWS_ERR_FORMAT;
  if (n < 0) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t) return GWS_ERR_NULL;
  for (int i = 0; i < n; ++i) {
    int rc = check_bwd(t[i]);
    if (rc != GWS_OK) return rc;
  }
  return run_batched(t, n, nullptr, nullptr, false, 0, step, (hipStream_t)stream, false, basis);
}

int gws_noise_basis(void* out, int64_t rows, int64_t cols, int64_t row0, int64_t col0, uint64_t seed, uint64_t step,
                    int basis, void* stream) {
  if (basis != GWS_BASIS_BITS && basis != GWS_BASIS_UNIFORM_BF16 && basis != GWS_BASIS_BOX_MULLER) return GWS_ERR_FORMAT;
  if (basis == GWS_BASIS_BITS) return GWS_ERR_FORMAT;   // the bit basis has its own, packed dump: gws_noise_packed
  if (rows < 0 || cols < 0 || row0 < 0 || col0 < 0 || (col0 & 7) != 0 || (cols & 7) != 0) return GWS_ERR_SHAPE;
  if (rows + row0 > (int64_t)0xFFFFFFFFll || (cols + col0) / 8 > (int64_t)0xFFFFFFFFll) return GWS_ERR_SHAPE;
  if (rows == 0 || cols == 0) return GWS_OK;
  if (!out) return GWS_ERR_NULL;
  if (!aligned(out, 16)) return GWS_ERR_ALIGN;
  const int64_t ngrp = cols / 8;
  if ((uint64_t)rows * (uint64_t)ngrp >= ((uint64_t)1 << 39)) return GWS_ERR_SHAPE;
  return launch_noise_basis(out, (uint32_t)rows, (uint32_t)ngrp, (uint32_t)row0, (uint32_t)(col0 / 8), seed, step, basis,
                            (hipStream_t)stream);
}

int gws_sample_bwd_tuned(const gws_tensor* t, int n, uint64_t step, int variant, int per_x, void* stream) {
  if (n < 0 || variant < -1 || variant > 1 || per_x < 0 || per_x > 64) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t) return GWS_ERR_NULL;
  for (int i = 0; i < n; ++i) {
    int rc = check_bwd(t[i]);
    if (rc != GWS_OK) return rc;
  }
  Tuning tune;
  tune.variant = variant;
  tune.per_x = per_x;
  return run_batched(t, n, nullptr, nullptr, false, 0, step, (hipStream_t)stream, false, kBasisBits, tune);
}

int gws_sample_fwd_tuned(const gws_tensor* t, int n, int fmt, uint64_t step, int variant, int per_x, void* stream) {
  if (n < 0 || variant < -1 || variant > 1 || per_x < 0 || per_x > 64) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t) return GWS_ERR_NULL;
  if (fmt != GWS_FMT_BF16 && fmt != GWS_FMT_FP8_E4M3 && fmt != GWS_FMT_FP6_E3M2) return GWS_ERR_FORMAT;
  for (int i = 0; i < n; ++i) {
    int rc = check_fwd(t[i]);
    if (rc != GWS_OK) return rc;
  }
  Tuning tune;
  tune.variant = variant;
  tune.per_x = per_x;
  return run_batched(t, n, nullptr, nullptr, true, fmt, step, (hipStream_t)stream, false, kBasisBits, tune);
}

int gws_copy_tiles(const gws_tensor* t, int n, void* stream) {
  if (n < 0) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t) return GWS_ERR_NULL;
  for (int i = 0; i < n; ++i) {
    int rc = check_shape(t[i]);
    if (rc != GWS_OK) return rc;
    if (t[i].rows == 0 || t[i].cols == 0) continue;
    if (!t[i].w || !t[i].w_hat) return GWS_ERR_NULL;
    if (!aligned(t[i].w, 16) || !aligned(t[i].w_hat, 16)) return GWS_ERR_ALIGN;
    if (overlap(t[i].w, t[i].w_hat, (size_t)t[i].rows * t[i].ld * 2)) return GWS_ERR_ALIAS;
  }
  return run_batched(t, n, nullptr, nullptr, true, kCopyOnly, 0, (hipStream_t)stream);
}

int gws_block_absmax(const gws_tensor* t, int n, void* stream) {
  if (n < 0) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t) return GWS_ERR_NULL;
  for (int i = 0; i < n; ++i) {
    int rc = check_shape(t[i]);
    if (rc != GWS_OK) return rc;
    if (t[i].rows == 0 || t[i].cols == 0) continue;
    if (!t[i].w || !t[i].scale) return GWS_ERR_NULL;
    if (!aligned(t[i].w, 16) || !aligned(t[i].scale, 4)) return GWS_ERR_ALIGN;
  }
  return run_batched(t, n, nullptr, nullptr, false, kAbsmaxOnly, 0, (hipStream_t)stream);
}

int gws_sample_fwd_bi(const gws_tensor* t, int n, const gws_bitwidth* bw, int fmt, uint64_t step, void* stream) {
  if (n < 0) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t || !bw) return GWS_ERR_NULL;
  if (fmt != GWS_FMT_BF16 && fmt != GWS_FMT_FP8_E4M3 && fmt != GWS_FMT_FP6_E3M2) return GWS_ERR_FORMAT;
  for (int i = 0; i < n; ++i) {
    int rc = check_fwd(t[i]);
    if (rc != GWS_OK) return rc;
  }
  return run_batched(t, n, bw, nullptr, true, fmt, step, (hipStream_t)stream);
}

int gws_sample_fwd_mx(const gws_tensor* t, const gws_mx_out* o, int n, int fmt, uint64_t step, void* stream) {
  if (n < 0) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t || !o) return GWS_ERR_NULL;
  if (fmt != GWS_FMT_FP8_E4M3 && fmt != GWS_FMT_FP6_E3M2) return GWS_ERR_FORMAT;
  for (int i = 0; i < n; ++i) {
    int rc = check_fwd_mx(t[i], o[i], fmt);
    if (rc != GWS_OK) return rc;
  }
  return run_batched(t, n, nullptr, o, true, fmt, step, (hipStream_t)stream);
}

int gws_sample_bwd_bi(const gws_tensor* t, int n, const gws_bitwidth* bw, uint64_t step, void* stream) {
  if (n < 0) return GWS_ERR_SHAPE;
  if (n == 0) return GWS_OK;
  if (!t || !bw) return GWS_ERR_NULL;
  for (int i = 0; i < n; ++i) {
    int rc = check_bwd(t[i]);
    if (rc != GWS_OK) return rc;
    if (bw[i].layer_blocks < 0) return GWS_ERR_SHAPE;
    if (t[i].rows == 0 || t[i].cols == 0) continue;
    if (!t[i].bt) return GWS_ERR_NULL;
    if (!aligned(t[i].bt, 4)) return GWS_ERR_ALIGN;
  }
  return run_batched(t, n, bw, nullptr, false, 0, step, (hipStream_t)stream);
}

int gws_noise_packed(void* out, int64_t rows, int64_t cols, int64_t row0, int64_t col0,
                     uint64_t seed, uint64_t step, void* stream) {
  if (rows < 0 || cols < 0 || row0 < 0 || col0 < 0 || (col0 & 7) != 0) return GWS_ERR_SHAPE;
  if (rows + row0 > (int64_t)0xFFFFFFFFll || (cols + col0) / 8 > (int64_t)0xFFFFFFFFll) return GWS_ERR_SHAPE;
  if (rows == 0 || cols == 0) return GWS_OK;
  if (!out) return GWS_ERR_NULL;
  if (!aligned(out, 4)) return GWS_ERR_ALIGN;
  const int64_t ngrp = (cols + 7) / 8;
  if ((uint64_t)rows * (uint64_t)ngrp >= ((uint64_t)1 << 39)) return GWS_ERR_SHAPE;
  return launch_noise_packed((uint32_t*)out, (uint32_t)rows, (uint32_t)ngrp, (uint32_t)row0,
                             (uint32_t)(col0 / 8), seed, step, (hipStream_t)stream);
}

int gws_linear_fwd_mode(const void* x, int64_t M, int64_t K, int64_t ldx, const gws_tensor* w, int w_is_nk,
                        int fmt, uint64_t step, void* y, int64_t ldy, int mode, void* stream) {
  if (!w) return GWS_ERR_NULL;
  if (fmt != GWS_FMT_BF16 && fmt != GWS_FMT_FP8_E4M3 && fmt != GWS_FMT_FP6_E3M2) return GWS_ERR_FORMAT;
  if (mode != GWS_LINEAR_AUTO && mode != GWS_LINEAR_IN_OPERAND && mode != GWS_LINEAR_TWO_KERNELS) return GWS_ERR_FORMAT;
  int rc = check_linear(x, M, K, ldx, w, w_is_nk, y, ldy);
  if (rc != GWS_OK || M == 0 || (w_is_nk ? w->rows : w->cols) == 0) return rc;
  if ((w->w_hat == nullptr) != (w->scale == nullptr)) return GWS_ERR_NULL;
  if (!aligned(w->w_hat, 16) || !aligned(w->scale, 4)) return GWS_ERR_ALIGN;
  if (w->w_hat && overlap(w->w, w->w_hat, (size_t)w->rows * w->ld * 2)) return GWS_ERR_ALIAS;
  GemmArgs g = linear_args(x, M, K, ldx, w, w_is_nk, step, y, ldy);
  g.scale = w->scale; g.w_hat = (uint16_t*)w->w_hat;
  if (mode == GWS_LINEAR_AUTO) {
    // Measured on MI355X: sampling the weight once with the streaming kernel and running the plain GEMM on
    // w_hat beats the kernel that samples in its operand load at every M (8192 tokens: 0.155 against 0.61 ms;
    // 16 .. 128 tokens: 28 .. 76 us against 40 .. 125 us for weights of 768 x 768 .. 2048 x 5632).
    mode = w->w_hat ? GWS_LINEAR_TWO_KERNELS : GWS_LINEAR_IN_OPERAND;
  }
  if (mode == GWS_LINEAR_TWO_KERNELS) {
    if (!w->w_hat) return GWS_ERR_NULL;
    rc = run_batched(w, 1, nullptr, nullptr, true, fmt, step, (hipStream_t)stream, /*keep=*/true);
    if (rc != GWS_OK) return rc;
    g.w = g.w_hat;
    return launch_gemm(g, w_is_nk, 0, GWS_FMT_BF16, (hipStream_t)stream);
  }
  return launch_gemm(g, w_is_nk, kFusedInOperand, fmt, (hipStream_t)stream);
}

size_t gws_linear_fwd_workspace_bytes(const gws_tensor* w) {
  if (!w || check_shape(*w) != GWS_OK || w->rows == 0 || w->cols == 0) return 0;
  return staged_bytes(*w) + (size_t)((w->rows + 31) / 32) * (size_t)((w->cols + 31) / 32) * sizeof(float);
}

int gws_linear_fwd_ws(const void* x, int64_t M, int64_t K, int64_t ldx, const gws_tensor* w, int w_is_nk,
                      int fmt, uint64_t step, void* y, int64_t ldy, void* workspace, size_t workspace_bytes,
                      void* stream) {
  if (!w) return GWS_ERR_NULL;
  if (fmt != GWS_FMT_BF16 && fmt != GWS_FMT_FP8_E4M3 && fmt != GWS_FMT_FP6_E3M2) return GWS_ERR_FORMAT;
  int rc = check_linear(x, M, K, ldx, w, w_is_nk, y, ldy);
  if (rc != GWS_OK || M == 0 || (w_is_nk ? w->rows : w->cols) == 0) return rc;
  if (!workspace) return GWS_ERR_NULL;
  if (!aligned(workspace, 256)) return GWS_ERR_ALIGN;
  if (workspace_bytes < gws_linear_fwd_workspace_bytes(w)) return GWS_ERR_SHAPE;
  return linear_staged(x, M, K, ldx, w, w_is_nk, fmt, step, y, ldy, workspace, (hipStream_t)stream);
}

int gws_linear_fwd_static(const void* x, int64_t M, int64_t K, int64_t ldx, const gws_tensor* w, int w_is_nk,
                          int fmt, uint64_t step, void* y, int64_t ldy, void* stream) {
  if (!w) return GWS_ERR_NULL;
  if (fmt != GWS_FMT_BF16 && fmt != GWS_FMT_FP8_E4M3 && fmt != GWS_FMT_FP6_E3M2) return GWS_ERR_FORMAT;
  int rc = check_linear(x, M, K, ldx, w, w_is_nk, y, ldy);
  if (rc != GWS_OK || M == 0 || (w_is_nk ? w->rows : w->cols) == 0) return rc;
  if (gws_linear_fwd_workspace_bytes(w) > (size_t)GWS_STATIC_SCRATCH_BYTES) return GWS_ERR_TOO_LARGE;
  void* staging = nullptr;
  rc = scratch_of_current_device(&staging);
  if (rc != GWS_OK) return rc;
  return linear_staged(x, M, K, ldx, w, w_is_nk, fmt, step, y, ldy, staging, (hipStream_t)stream);
}

int gws_linear_fwd(const void* x, int64_t M, int64_t K, int64_t ldx, const gws_tensor* w, int w_is_nk,
                   int fmt, uint64_t step, void* y, int64_t ldy, void* stream) {
  return gws_linear_fwd_mode(x, M, K, ldx, w, w_is_nk, fmt, step, y, ldy, GWS_LINEAR_AUTO, stream);
}

// Arguments of the weight-gradient GEMM checked and put into the GEMM's terms.
static int bwd_w_args(const void* x, const void* dy, int64_t M, int64_t ldx, int64_t ldy, const gws_tensor* w, int w_is_nk,
                      uint64_t step, GemmArgs& g) {
  if (!w) return GWS_ERR_NULL;
  int rc = check_shape(*w);
  if (rc != GWS_OK) return rc;
  const int64_t K = w_is_nk ? w->cols : w->rows, N = w_is_nk ? w->rows : w->cols;
  if (M <= 0 || M >= (int64_t)1 << 31 || (M & 63) != 0) return GWS_ERR_SHAPE;
  if (w->rows <= 0 || w->cols <= 0 || (w->rows & 255) != 0 || (w->cols & 255) != 0) return GWS_ERR_SHAPE;
  if (ldx < K || ldy < N || (ldx & 7) != 0 || (ldy & 7) != 0 || ldx >= (int64_t)1 << 31 || ldy >= (int64_t)1 << 31) return GWS_ERR_SHAPE;
  if (!x || !dy || !w->dw) return GWS_ERR_NULL;
  if (w->dbt && !w->scale) return GWS_ERR_NULL;
  if (!aligned(x, 16) || !aligned(dy, 16) || !aligned(w->dw, 16) || !aligned(w->dbt, 4) || !aligned(w->scale, 4)) return GWS_ERR_ALIGN;
  const size_t dw_bytes = (size_t)w->rows * w->ld * 2;
  if (overlap2(w->dw, dw_bytes, x, (size_t)M * ldx * 2) || overlap2(w->dw, dw_bytes, dy, (size_t)M * ldy * 2)) return GWS_ERR_ALIAS;
  memset(&g, 0, sizeof g);
  // C[rows x cols] = A^T B over the M tokens: A supplies the rows of the stored weight
  g.x = (const uint16_t*)(w_is_nk ? dy : x); g.ldx = (uint32_t)(w_is_nk ? ldy : ldx);
  g.w = (const uint16_t*)(w_is_nk ? x : dy); g.ldw = (uint32_t)(w_is_nk ? ldx : ldy);
  g.y = (uint16_t*)w->dw; g.ldy = (uint32_t)w->ld;
  g.M = (uint32_t)w->rows; g.N = (uint32_t)w->cols; g.K = (uint32_t)M;
  g.scale = w->scale; g.dbt = w->dbt;
  g.row0 = (uint32_t)w->row0; g.cg0 = (uint32_t)(w->col0 / 8);
  g.seed_lo = (uint32_t)w->seed; g.seed_hi = (uint32_t)(w->seed >> 32);
  g.step_lo = (uint32_t)step; g.step_hi = (uint32_t)(step >> 32);
  return gemm256_tn_applicable(g) ? GWS_OK : GWS_ERR_SHAPE;
}

// Into how many parts the tokens are split so that a weight of few 256 x 256 tiles still fills the chip: as many
// as keep all workgroups in one round, at least 8 K-steps of 64 tokens each, at most 8 (every part costs a pass
// over an fp32 copy of the gradient in the second kernel).
static uint32_t bwd_w_parts(int64_t rows, int64_t cols, int64_t M) {
  const int64_t tiles = (rows / 256) * (cols / 256);
  const int cus = compute_units();
  if (tiles <= 0 || cus <= 0) return 1;
  int64_t parts = cus / tiles;
  if (parts > 8) parts = 8;
  if (parts > M / 64 / 8) parts = M / 64 / 8;
  return parts < 2 ? 1u : (uint32_t)parts;
}

int gws_linear_bwd_w(const void* x, const void* dy, int64_t M, int64_t ldx, int64_t ldy, const gws_tensor* w,
                     int w_is_nk, uint64_t step, void* stream) {
  GemmArgs g;
  const int rc = bwd_w_args(x, dy, M, ldx, ldy, w, w_is_nk, step, g);
  if (rc != GWS_OK) return rc;
  return launch_gemm256_tn(g, w->dbt != nullptr, (hipStream_t)stream);
}

size_t gws_linear_bwd_w_workspace_bytes(const gws_tensor* w, int64_t M) {
  if (!w || w->rows <= 0 || w->cols <= 0 || (w->rows & 255) != 0 || (w->cols & 255) != 0 || M <= 0 || (M & 63) != 0) return 0;
  const uint32_t parts = bwd_w_parts(w->rows, w->cols, M);
  return parts < 2 ? 0 : (size_t)parts * (size_t)(w->rows / 256) * (size_t)(w->cols / 256) * 256 * 256 * sizeof(float);
}

int gws_linear_bwd_w_ws(const void* x, const void* dy, int64_t M, int64_t ldx, int64_t ldy, const gws_tensor* w,
                        int w_is_nk, uint64_t step, void* workspace, size_t workspace_bytes, void* stream) {
  GemmArgs g;
  const int rc = bwd_w_args(x, dy, M, ldx, ldy, w, w_is_nk, step, g);
  if (rc != GWS_OK) return rc;
  uint32_t parts = bwd_w_parts(w->rows, w->cols, M);
  const size_t per_part = gemm256_tn_split_bytes(g, 1);
  if (workspace == nullptr) workspace_bytes = 0;
  if (parts > workspace_bytes / per_part) parts = (uint32_t)(workspace_bytes / per_part);   // as many parts as the workspace holds
  if (parts < 2) return launch_gemm256_tn(g, w->dbt != nullptr, (hipStream_t)stream);
  if (!aligned(workspace, 16)) return GWS_ERR_ALIGN;
  const size_t ws_bytes = gemm256_tn_split_bytes(g, parts);
  if (overlap2(workspace, ws_bytes, w->dw, (size_t)w->rows * w->ld * 2) || overlap2(workspace, ws_bytes, x, (size_t)M * ldx * 2) ||
      overlap2(workspace, ws_bytes, dy, (size_t)M * ldy * 2)) return GWS_ERR_ALIAS;
  return launch_gemm256_tn_split(g, w->dbt != nullptr, (float*)workspace, parts, (hipStream_t)stream);
}

int gws_gemm_bf16(const void* x, int64_t M, int64_t K, int64_t ldx, const void* w, int64_t N, int64_t ldw,
                  int w_is_nk, void* y, int64_t ldy, void* stream) {
  if (M < 0 || K < 0 || N < 0 || M >= (int64_t)1 << 31 || N >= (int64_t)1 << 31 || K >= (int64_t)1 << 31) return GWS_ERR_SHAPE;
  if (M == 0 || N == 0) return GWS_OK;
  if ((K & 31) != 0 || (N & 31) != 0 || K == 0) return GWS_ERR_SHAPE;
  const int64_t wcols = w_is_nk ? K : N;
  if (ldx < K || ldy < N || ldw < wcols || ((ldx | ldy | ldw) & 7) != 0 ||
      ldx >= (int64_t)1 << 31 || ldy >= (int64_t)1 << 31 || ldw >= (int64_t)1 << 31) return GWS_ERR_SHAPE;
  if (!x || !w || !y) return GWS_ERR_NULL;
  if (!aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16)) return GWS_ERR_ALIGN;
  GemmArgs g;
  memset(&g, 0, sizeof g);
  g.x = (const uint16_t*)x; g.w = (const uint16_t*)w; g.y = (uint16_t*)y;
  g.M = (uint32_t)M; g.N = (uint32_t)N; g.K = (uint32_t)K;
  g.ldx = (uint32_t)ldx; g.ldw = (uint32_t)ldw; g.ldy = (uint32_t)ldy;
  return launch_gemm(g, w_is_nk, 0, GWS_FMT_BF16, (hipStream_t)stream);
}

// How many of the weights next[0 .. n_next) ride in the launch of the GEMM g (a prefix of the list), with the riders'
// descriptors, the number of extra workgroups and the riding loop to use.
// Ride along when the 256-tile GEMM leaves compute units without a tile in its last round and the sampling fits
// beside that round.  Measured on MI355X: a riding wavefront (one per SIMD, the GEMM's register allocation) takes
// about 1.8 us per 32 x 64 tile in ride_tiles and 2.1 us in sample_tiles; a GEMM tile about 1.5 us per K-step of 64.
static int plan_ride(const GemmArgs& g, bool gemm_empty, int64_t K, const gws_tensor* next, int n_next, int force_extra,
                     int rider, RideList& r, uint32_t& idle, int& use_rider) {
  memset(&r, 0, sizeof r);
  idle = 0;
  use_rider = 1;
  const bool gemm_rides = force_extra >= 0 ? (gemm_empty || gemm256_applicable(g)) : (!gemm_empty && gemm256_applicable(g));
  if (!gemm_rides) return 0;
  const int cus = compute_units();
  const uint64_t tiles = gemm_empty ? 0 : (uint64_t)(g.M / 256) * (uint64_t)(g.N / 256);
  idle = cus > 0 ? (uint32_t)((cus - tiles % cus) % cus) : 0u;
  if (force_extra >= 0) idle = (uint32_t)force_extra;
  if (idle == 0) return 0;
  const double t_tile_us = (double)(K / 64) * 1.5 + 5.0;
  int n_riding = 0;
  double t_sample_us = 0.0;
  uint32_t begin = 0;
  for (int i = 0; i < n_next && n_riding < kMaxRide; ++i) {
    const gws_tensor& t = next[i];
    if (t.rows == 0 || t.cols == 0 || (t.rows & 31) != 0 || (t.cols & 63) != 0) break;
    const bool wide = (t.cols & 255) == 0 && rider != 0;
    if (!wide && i > 0) break;                                                      // sample_tiles takes one weight
    const double units = (double)(t.rows / 32) * (double)(t.cols / 64);             // wavefront tiles
    const double add = units / (4.0 * idle) * (wide ? 1.8 : 2.1);
    // with a margin: a riding part that outlasts the tiles costs more than the launch it saves
    if (force_extra < 0 && t_sample_us + add > (wide ? 0.8 : 0.6) * t_tile_us) break;
    t_sample_us += add;
    TileDesc& d = r.d[n_riding];
    memset(&d, 0, sizeof d);
    d.p0 = t.w; d.p1 = t.w_hat; d.p2 = (void*)t.bt; d.p3 = t.scale; d.p4 = nullptr;
    fill_common(d, t, 1);
    d.b_target = 0.0f; d.b_delta = 1.0f; d.lambda_m = 0.0f;
    d.first_wg = begin;
    r.begin[n_riding] = begin;
    begin += (uint32_t)((t.rows / 32) * (t.cols / 256));
    ++n_riding;
    if (!wide) {
      use_rider = 0;
      break;
    }
  }
  for (int j = n_riding; j <= kMaxRide; ++j) r.begin[j] = begin;
  r.n = (uint32_t)n_riding;
  return n_riding;
}

// The plain GEMM with the forward sampling of `n_next` weights: as many of them as fit ride in the GEMM's launch
// (in the order given), the others are sampled by one launch of the sampling kernel after it.
// force_extra >= 0: ride with that many extra workgroups whatever the estimate says (measurement); rider: the riding
// loop (launch_gemm256_ride), -1 = the library's choice.
static int gemm_sample_next(const void* x, int64_t M, int64_t K, int64_t ldx, const void* w, int64_t N, int64_t ldw,
                            int w_is_nk, void* y, int64_t ldy, const gws_tensor* next, int n_next, int fmt, uint64_t step,
                            int force_extra, int rider, void* stream) {
  if (n_next < 0 || n_next > 64) return GWS_ERR_SHAPE;
  if (n_next == 0) return gws_gemm_bf16(x, M, K, ldx, w, N, ldw, w_is_nk, y, ldy, stream);
  if (!next) return GWS_ERR_NULL;
  if (fmt != GWS_FMT_BF16 && fmt != GWS_FMT_FP8_E4M3 && fmt != GWS_FMT_FP6_E3M2) return GWS_ERR_FORMAT;
  for (int i = 0; i < n_next; ++i) {
    int rc = check_fwd(next[i]);
    if (rc != GWS_OK) return rc;
  }
  // the GEMM's own argument rules (as gws_gemm_bf16), checked before anything is launched
  if (M < 0 || K < 0 || N < 0 || M >= (int64_t)1 << 31 || N >= (int64_t)1 << 31 || K >= (int64_t)1 << 31) return GWS_ERR_SHAPE;
  const bool gemm_empty = (M == 0 || N == 0);
  if (!gemm_empty) {
    if ((K & 31) != 0 || (N & 31) != 0 || K == 0) return GWS_ERR_SHAPE;
    const int64_t wcols = w_is_nk ? K : N;
    if (ldx < K || ldy < N || ldw < wcols || ((ldx | ldy | ldw) & 7) != 0 ||
        ldx >= (int64_t)1 << 31 || ldy >= (int64_t)1 << 31 || ldw >= (int64_t)1 << 31) return GWS_ERR_SHAPE;
    if (!x || !w || !y) return GWS_ERR_NULL;
    if (!aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16)) return GWS_ERR_ALIGN;
    // a sampled weight must not be an operand or the result of this GEMM
    for (int i = 0; i < n_next; ++i) {
      const size_t hat_bytes = (size_t)next[i].rows * next[i].ld * 2;
      if (next[i].rows > 0 && next[i].cols > 0 &&
          (overlap2(next[i].w_hat, hat_bytes, w, (size_t)(w_is_nk ? N : K) * ldw * 2) ||
           overlap2(next[i].w_hat, hat_bytes, x, (size_t)M * ldx * 2) || overlap2(next[i].w_hat, hat_bytes, y, (size_t)M * ldy * 2)))
        return GWS_ERR_ALIAS;
    }
  }
  GemmArgs g;
  memset(&g, 0, sizeof g);
  g.x = (const uint16_t*)x; g.w = (const uint16_t*)w; g.y = (uint16_t*)y;
  g.M = (uint32_t)M; g.N = (uint32_t)N; g.K = (uint32_t)K;
  g.ldx = (uint32_t)ldx; g.ldw = (uint32_t)ldw; g.ldy = (uint32_t)ldy;
  if (gemm_empty) g.M = g.N = 0;

  RideList r;
  uint32_t idle = 0;
  int use_rider = 1;
  const int n_riding = plan_ride(g, gemm_empty, K, next, n_next, force_extra, rider, r, idle, use_rider);   // the first n_riding ride
  if (n_riding > 0) {
    int rc = launch_gemm256_ride(g, w_is_nk, r, fmt, step, idle, use_rider, (hipStream_t)stream);
    if (rc != GWS_OK) return rc;
  }
  if (n_riding == 0 && !gemm_empty) {
    int rc = launch_gemm(g, w_is_nk, 0, GWS_FMT_BF16, (hipStream_t)stream);
    if (rc != GWS_OK) return rc;
  }
  if (n_riding == n_next) return GWS_OK;
  return run_batched(next + n_riding, n_next - n_riding, nullptr, nullptr, true, fmt, step, (hipStream_t)stream, /*keep=*/true);
}

int gws_gemm_bf16_sample_next(const void* x, int64_t M, int64_t K, int64_t ldx, const void* w, int64_t N, int64_t ldw,
                              int w_is_nk, void* y, int64_t ldy, const gws_tensor* next, int fmt, uint64_t step,
                              void* stream) {
  return gemm_sample_next(x, M, K, ldx, w, N, ldw, w_is_nk, y, ldy, next, next ? 1 : 0, fmt, step, -1, -1, stream);
}

int gws_gemm_bf16_sample_next_n(const void* x, int64_t M, int64_t K, int64_t ldx, const void* w, int64_t N, int64_t ldw,
                                int w_is_nk, void* y, int64_t ldy, const gws_tensor* next, int n_next, int fmt,
                                uint64_t step, void* stream) {
  return gemm_sample_next(x, M, K, ldx, w, N, ldw, w_is_nk, y, ldy, next, n_next, fmt, step, -1, -1, stream);
}

int gws_ride_plan(int64_t M, int64_t K, int64_t N, const gws_tensor* next, int n_next) {
  if (!next || n_next <= 0 || M <= 0 || N <= 0 || K <= 0) return 0;
  GemmArgs g;
  memset(&g, 0, sizeof g);
  g.M = (uint32_t)M; g.N = (uint32_t)N; g.K = (uint32_t)K;
  RideList r;
  uint32_t idle = 0;
  int use_rider = 1;
  return plan_ride(g, false, K, next, n_next, -1, -1, r, idle, use_rider);
}

int gws_gemm_bf16_ride_probe(const void* x, int64_t M, int64_t K, int64_t ldx, const void* w, int64_t N, int64_t ldw,
                             int w_is_nk, void* y, int64_t ldy, const gws_tensor* next, int fmt, uint64_t step,
                             int extra_workgroups, int rider, void* stream) {
  if (!next || extra_workgroups < 1 || extra_workgroups > 4096 || rider < 0 || rider > 1) return GWS_ERR_SHAPE;
  if ((next->rows & 31) != 0 || (next->cols & 63) != 0) return GWS_ERR_SHAPE;
  return gemm_sample_next(x, M, K, ldx, w, N, ldw, w_is_nk, y, ldy, next, 1, fmt, step, extra_workgroups, rider, stream);
}

// Philox4x32-10 on the host, for the seed derivation only.
uint64_t gws_derive_seed(uint64_t user_seed, uint64_t tensor_id) {
  uint32_t c0 = (uint32_t)tensor_id, c1 = (uint32_t)(tensor_id >> 32), c2 = 0x47575331u, c3 = 0u;
  uint32_t k0 = (uint32_t)user_seed, k1 = (uint32_t)(user_seed >> 32);
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return (uint64_t)c0 | ((uint64_t)c1 << 32);
}

const char* gws_status_string(int status) {
  switch (status) {
    case GWS_OK: return "ok";
    case GWS_ERR_NULL: return "required pointer is NULL";
    case GWS_ERR_SHAPE: return "invalid shape, leading dimension or shard origin";
    case GWS_ERR_ALIGN: return "misaligned pointer";
    case GWS_ERR_FORMAT: return "unknown target format";
    case GWS_ERR_LAUNCH: return "kernel launch failed";
    case GWS_ERR_ALIAS: return "output overlaps input";
    case GWS_ERR_TOO_LARGE: return "operand exceeds a fixed capacity of the library";
    default: return "unknown status";
  }
}

int gws_version(void) { return 7; }

}  // extern "C"
