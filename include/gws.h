/*
 * libgws -- Gaussian weight sampling (GaussWS) hot path for AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer named "device" is HIP device memory owned by the caller;
 * every other pointer is host memory.  The library allocates no device memory,
 * keeps no global state (one exception is stated at gws_linear_fwd_static) and is
 * thread-safe.  All GPU work is enqueued
 * asynchronously on the given stream (a hipStream_t passed as void*, NULL = the
 * default stream); no call synchronises.
 * The return value is a gws_status and reports argument and launch errors only;
 * on any error nothing has been launched for the failing call.
 *
 * Notation follows the paper: w is a BF16 weight matrix [rows x cols], split in
 * square blocks of b_l = 32; b_t is the per-block bitwidth; R is the noise basis
 * approximating round(N(0,1)/2); w_hat is the sampled weight.
 *
 * Noise identity between forward and backward (paper Sec. 3.5 "GPU memory",
 * Sec. 3.6 "Managing seed"): R is a pure function of (seed, step, row, column),
 * so a backward call with the seed and step of the forward call regenerates the
 * same R and no noise tensor is ever stored.  The 16 random bits of element
 * (i, j) are one nibble of each of the four words of
 *   Philox4x32-10(counter = (col0/8 + j>>3, row0 + i, step_lo, step_hi),
 *                 key     = (seed_lo, seed_hi)),
 * namely nibble (k >> 1) + 4 * (k & 1) with k = j & 7: even elements of a group of
 * eight read the low 16-bit half of each word, odd elements the high half.
 */
#ifndef GWS_H
#define GWS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GWS_BLOCK 32 /* b_l, paper Sec. 3.2 */

/* Target format fp_{e,m} of the cast that follows the addition (paper Sec. 3.3).
 * The cast is block-scaled (MX style): with Ea = floor(log2 max|w|) of the block,
 * values are rounded (nearest, ties to even, gradual underflow, saturating) to
 * X * {codes of the format}, X = 2^(Ea + 1 - emax), which puts the format's top
 * binade on the headroom binade that w_hat can reach (proof of Prop. 3).
 * The result is stored in a BF16 container (2 bytes per parameter, Sec. 3.5). */
typedef enum gws_format {
  GWS_FMT_BF16 = 0,     /* no further rounding after the BF16 add             */
  GWS_FMT_FP8_E4M3 = 1, /* OCP FP8 E4M3: emax 8, emin -6, 3 mantissa bits, max 448 */
  GWS_FMT_FP6_E3M2 = 2  /* OCP MX FP6 E3M2: emax 4, emin -2, 2 mantissa bits, max 28 */
} gws_format;

typedef enum gws_status {
  GWS_OK = 0,
  GWS_ERR_NULL = 1,   /* a required pointer is NULL                              */
  GWS_ERR_SHAPE = 2,  /* negative size, ld < cols, ld % 8 != 0, size >= 2^31,
                         row0/col0 not a multiple of 32, n < 0                   */
  GWS_ERR_ALIGN = 3,  /* BF16 pointer not 16-byte aligned, fp32 pointer not 4-byte */
  GWS_ERR_FORMAT = 4, /* unknown gws_format                                      */
  GWS_ERR_LAUNCH = 5, /* the HIP runtime refused a kernel launch                 */
  GWS_ERR_ALIAS = 6,  /* an output overlaps an input it must not overlap         */
  GWS_ERR_TOO_LARGE = 7 /* the operand exceeds a fixed capacity of the library (gws_linear_fwd_static) */
} gws_status;

/* One weight tensor, row-major.  BF16 buffers are [rows x ld] with ld >= cols
 * elements per row (ld a multiple of 8, base 16-byte aligned); columns >= cols
 * of an output row are never written.  Per-block fp32 buffers are
 * [ceil(rows/32) x ceil(cols/32)] row-major, dense.  rows or cols may be 0 (the
 * tensor is then skipped) and need not be multiples of 32: an edge block holds
 * only the elements that exist.                                                   */
typedef struct gws_tensor {
  const void* w;      /* device, BF16: weight (forward in)                        */
  void* w_hat;        /* device, BF16: sampled weight (forward out); not w        */
  const float* bt;    /* device, fp32 per block: bitwidth b_t (forward in)        */
  float* scale;       /* device, fp32 per block: max|w| * 2^(1-b_t), unrounded
                         fp32 (forward out, backward in)                          */
  const void* g;      /* device, BF16: dL/dw_hat (backward in)                    */
  void* dw;           /* device, BF16: dL/dw (backward out).  NULL or == g: the
                         pass-through is an alias and nothing is copied           */
  float* dbt;         /* device, fp32 per block: dL/db_t (backward out)           */
  int64_t rows, cols; /* elements                                                 */
  int64_t ld;         /* leading dimension of w, w_hat, g, dw (elements)          */
  int64_t row0, col0; /* position of this tensor inside a larger, sharded tensor
                         (multiples of 32; 0 for a whole tensor).  They only
                         enter the noise counter, so shards reproduce the noise
                         of the unsharded tensor                                  */
  uint64_t seed;      /* per-tensor seed, see gws_derive_seed                     */
} gws_tensor;

/* Forward, paper Eq. 3 followed by the cast of Sec. 3.3, for n tensors in as few
 * launches as possible:
 *   a      = max_{b_l}|w|                                  (exact)
 *   s32    = fp32(a) * 2^(1 - b_t)                         (fp32; 2^t is the
 *            library's fixed degree-6 polynomial, exact for integer t)
 *   s      = bf16_rne(s32)
 *   w_hat  = cast_fmt( bf16_rne( w + R * s ) )
 * where R * s is formed in sign-magnitude (R = -0 gives -0.0).  Writes w_hat and
 * scale (= s32).  `t` is a host array of n descriptors; it is read before the
 * call returns.  Uses fields w, w_hat, bt, scale, rows, cols, ld, row0, col0, seed. */
int gws_sample_fwd(const gws_tensor* t, int n, int fmt, uint64_t step, void* stream);

/* Backward, paper Eq. 4, for n tensors:
 *   dL/dw   = dL/dw_hat           (bit copy into dw unless dw is NULL or == g)
 *   dL/db_t = -ln2 * s32 * sum_{b_l}( dL/dw_hat .* R )      (fp32, fixed order)
 * with R regenerated from (seed, step) and s32 read from `scale` as the forward
 * call left it.  Uses fields g, dw, dbt, scale, rows, cols, ld, row0, col0, seed. */
int gws_sample_bwd(const gws_tensor* t, int n, uint64_t step, void* stream);

/* Bitwidth parametrisation of the paper's Sec. 3.6 "Bitwidth": every block keeps
 * an internal parameter b_i (initialised to 1) and
 *   b_t = b_target + b_i * (b_init - b_target)                          (Eq. 11)
 * and the training loss may carry the term
 *   lambda * sum_layers( sum_blocks |b_t - b_target| / m )              (Eq. 12)
 * with m the number of blocks of the layer.  One gws_bitwidth per tensor (host).   */
typedef struct gws_bitwidth {
  float b_init;          /* bitwidth at b_i = 1                                     */
  float b_target;        /* bitwidth at b_i = 0                                     */
  float lambda;          /* weight of the loss term of Eq. 12; 0 = no such term     */
  int64_t layer_blocks;  /* m of Eq. 12: blocks of the whole layer this tensor is, or
                            is a shard of; 0 = the tensor's own block count         */
} gws_bitwidth;

/* gws_sample_fwd with the bitwidth given through b_i: the field `bt` of every
 * descriptor holds b_i (device, fp32 per block) and the block uses
 *   b_t = fl( b_target + fl( b_i * fl(b_init - b_target) ) )            (fp32)
 * Everything else is gws_sample_fwd.  bw is a host array of n.                     */
int gws_sample_fwd_bi(const gws_tensor* t, int n, const gws_bitwidth* bw, int fmt, uint64_t step,
                      void* stream);

/* gws_sample_bwd for the parametrised bitwidth: writes, into the field `dbt`,
 *   dL'/db_i = (b_init - b_target) * ( dL/db_t + lambda / m * sgn(b_t - b_target) )
 * with dL/db_t as in gws_sample_bwd, b_t recomputed from b_i (field `bt`, required
 * here) as the forward call formed it, and sgn(0) = 0.  fp32.                       */
int gws_sample_bwd_bi(const gws_tensor* t, int n, const gws_bitwidth* bw, uint64_t step, void* stream);

/* The sampled weight as microscaling (MX) data, the deployment form of the formats
 * the paper targets (Sec. 3.1; with square blocks the same bytes serve W and its
 * transpose): per 32x32 block one E8M0 byte, the biased exponent of the cast's scale
 * X = 2^(xscale - 127), and per element the code of q / X in the element format,
 * where q is the value gws_sample_fwd stores in its BF16 container:
 *   q[i][j] == X(block of i, j) * value(code[i][j])      exactly.
 * FP8-E4M3 (bias 7; the NaN pattern S.1111.111 is never produced): one byte per
 * element, row i at codes + i * ldc.  FP6-E3M2 (bias 3): element j of row i occupies
 * bits [6j, 6j + 6) of the bytes at codes + i * ldc read as a little-endian bit
 * string (8 elements = 6 bytes; unused bits of a row's last byte are written as 0).
 * An all-zero block gets xscale = 127.  Bytes past a row's data are never written.  */
typedef struct gws_mx_out {
  void* codes;      /* device; 8-byte aligned for FP8, 2-byte aligned for FP6            */
  uint8_t* xscale;  /* device, [ceil(rows/32) x ceil(cols/32)] bytes                     */
  int64_t ldc;      /* bytes per row of codes: >= cols and a multiple of 8 (FP8),
                       >= ceil(cols * 6 / 8) and a multiple of 2 (FP6)                   */
} gws_mx_out;

/* gws_sample_fwd with MX output: for tensor i writes o[i].codes, o[i].xscale and
 * t[i].scale (the backward pass needs it); t[i].w_hat is not used.  fmt is
 * GWS_FMT_FP8_E4M3 or GWS_FMT_FP6_E3M2.  o is a host array of n.                      */
int gws_sample_fwd_mx(const gws_tensor* t, const gws_mx_out* o, int n, int fmt, uint64_t step,
                      void* stream);

/* Sampled-weight linear: Y = X * w_hat with w_hat produced as in gws_sample_fwd (the
 * paper, Sec. 3.5 "Separate kernels", keeps sampling and matmul apart; the fused kernels
 * here are the alternative, and the call picks whichever is faster).
 *   x : device BF16 [M x K], leading dimension ldx
 *   w : one descriptor (host).  w->w is [K x N] (rows = K, cols = N) or, when
 *       w_is_nk != 0, [N x K] (rows = N, cols = K; Y = X * w_hat^T).
 *       w->w_hat and w->scale are written if non-NULL (both or neither).
 *   y : device BF16 [M x N], leading dimension ldy; fp32 accumulation, one
 *       round-to-nearest-even to BF16.
 * K and N must be multiples of 32; ldx, ldy multiples of 8.
 * Two ways to the same bytes (w_hat, scale and Y are bit-identical between them):
 *   GWS_LINEAR_IN_OPERAND   one kernel; the sampling sits in the weight operand load of every
 *                           output tile (no w_hat round trip; each block is resampled once per
 *                           128 rows of X).  Any shape; w_hat/scale optional.
 *   GWS_LINEAR_TWO_KERNELS  the sampling kernel of gws_sample_fwd, then the plain GEMM on w_hat.
 *                           Needs w_hat/scale (GWS_ERR_NULL otherwise).
 *   GWS_LINEAR_AUTO         two kernels when w_hat/scale are given (the faster choice at every M
 *                           as measured on MI355X), else in-operand.
 * (Mode value 1 belonged to a retired kernel and is rejected with GWS_ERR_FORMAT.)
 * gws_linear_fwd is gws_linear_fwd_mode with GWS_LINEAR_AUTO.                              */
#define GWS_LINEAR_AUTO 0
#define GWS_LINEAR_IN_OPERAND 2
#define GWS_LINEAR_TWO_KERNELS 3
int gws_linear_fwd(const void* x, int64_t M, int64_t K, int64_t ldx,
                   const gws_tensor* w, int w_is_nk, int fmt, uint64_t step,
                   void* y, int64_t ldy, void* stream);
int gws_linear_fwd_mode(const void* x, int64_t M, int64_t K, int64_t ldx,
                        const gws_tensor* w, int w_is_nk, int fmt, uint64_t step,
                        void* y, int64_t ldy, int mode, void* stream);

/* gws_linear_fwd for a caller that wants Y only and many rows of X (Sec. 3.5 keeps sampling and
 * matmul apart; so does this): w_hat and scale are staged in `workspace` instead of the caller's
 * buffers (w->w_hat and w->scale are not used), then the plain GEMM runs on the staged w_hat.
 * Y is bit-identical to gws_linear_fwd's.
 *   workspace       : device, 256-byte aligned, owned by the caller; contents undefined afterwards;
 *                     must not overlap x, y or w->w (GWS_ERR_ALIAS)
 *   workspace_bytes : at least gws_linear_fwd_workspace_bytes(w) (GWS_ERR_SHAPE otherwise)
 * gws_linear_fwd_workspace_bytes: rows * ld * 2 rounded up to 256, plus 4 bytes per block; 0 for an
 * empty or invalid descriptor.  Host function, no GPU work.                                      */
size_t gws_linear_fwd_workspace_bytes(const gws_tensor* w);
int gws_linear_fwd_ws(const void* x, int64_t M, int64_t K, int64_t ldx,
                      const gws_tensor* w, int w_is_nk, int fmt, uint64_t step,
                      void* y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* gws_linear_fwd_ws for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It allocates
 * nothing and takes no workspace: w_hat and scale are staged in a buffer of GWS_STATIC_SCRATCH_BYTES
 * that is part of the loaded library (every GPU the library runs on holds its own copy until the
 * process ends; its address on a GPU is looked up on the first call made with that GPU current).
 * Same arguments, same results (Y bit-identical) as gws_linear_fwd_ws.
 *   - a weight with gws_linear_fwd_workspace_bytes(w) > GWS_STATIC_SCRATCH_BYTES is rejected with
 *     GWS_ERR_TOO_LARGE and nothing is launched;
 *   - all calls on one GPU share that GPU's buffer, which keeps the last call's contents: calls
 *     that overlap in time on one GPU (different streams, or threads) race on it; calls on one
 *     stream are ordered and safe.  This is the library's only state.                          */
#define GWS_STATIC_SCRATCH_BYTES (32u << 20)
int gws_linear_fwd_static(const void* x, int64_t M, int64_t K, int64_t ldx,
                          const gws_tensor* w, int w_is_nk, int fmt, uint64_t step,
                          void* y, int64_t ldy, void* stream);

/* Weight gradient of the sampled-weight linear with the reduction of Eq. 4 in the GEMM's
 * epilogue (the linear's backward pass, paper Eq. 2, applied to w_hat):
 *   dW      = X^T * dY                 fp32 accumulation, one round-to-nearest-even to BF16
 *   dL/db_t = -ln2 * s32 * sum_{b_l}( dW .* R )        on the rounded BF16 dW, fp32
 * so that dL/db_t costs no second pass over dW.  (dX = dY * w_hat^T is gws_gemm_bf16 on
 * w_hat with the other layout flag.)
 *   x  : device BF16 [M x K] (ldx), the linear's input;  dy : device BF16 [M x N] (ldy)
 *   w  : one descriptor (host) of the weight as stored: [K x N] (rows = K, cols = N) or,
 *        when w_is_nk != 0, [N x K].  Fields used: dw (out, required, [rows x ld]),
 *        dbt (out; NULL = plain GEMM), scale (in, required with dbt), rows, cols, ld,
 *        row0, col0, seed.
 * rows and cols must be multiples of 256, M a multiple of 64 and ldx, ldy below 2^28
 * (GWS_ERR_SHAPE otherwise);
 * M == 0 is an error, since dW would be undefined.  Given the same dW bytes,
 * gws_sample_bwd returns the same dL/db_t up to the order of the fp32 additions.        */
int gws_linear_bwd_w(const void* x, const void* dy, int64_t M, int64_t ldx, int64_t ldy,
                     const gws_tensor* w, int w_is_nk, uint64_t step, void* stream);

/* gws_linear_bwd_w for weights of few 256 x 256 tiles (a 2048 x 2048 weight has 64, on a part
 * with 256 compute units): the M tokens are split into parts, each part's workgroups leave an
 * fp32 partial tile in `workspace`, and a second kernel adds a tile's parts in a fixed order,
 * rounds once to BF16 and writes dW and dL/db_t as above.  Same arguments, results within the
 * same bounds (the fp32 additions are grouped by part; nothing depends on timing).
 *   gws_linear_bwd_w_workspace_bytes(w, M): bytes the split would use for this weight and M
 *     (host call; 0 when the one-kernel form is used: enough tiles, M too small, bad shape).
 *   workspace : device memory, 16-byte aligned, workspace_bytes long, not overlapping x, dy or
 *     dw (GWS_ERR_ALIGN / GWS_ERR_ALIAS); the library's only use of it is during this call's
 *     kernels, its contents afterwards are unspecified.  With less than
 *     gws_linear_bwd_w_workspace_bytes the tokens are split into as many parts as fit, with
 *     room for fewer than two parts (or workspace NULL) this is gws_linear_bwd_w.            */
size_t gws_linear_bwd_w_workspace_bytes(const gws_tensor* w, int64_t M);
int gws_linear_bwd_w_ws(const void* x, const void* dy, int64_t M, int64_t ldx, int64_t ldy,
                        const gws_tensor* w, int w_is_nk, uint64_t step,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Plain BF16 GEMM with the same tiling as gws_linear_fwd and no sampling:
 * Y = X * W (or X * W^T when w_is_nk).  The reference point the fused kernel's
 * overhead is measured against.  w is device BF16 with leading dimension ldw.     */
int gws_gemm_bf16(const void* x, int64_t M, int64_t K, int64_t ldx,
                  const void* w, int64_t N, int64_t ldw, int w_is_nk,
                  void* y, int64_t ldy, void* stream);

/* gws_gemm_bf16 with the forward sampling of another weight riding along: Y = X * W as above (W is
 * typically a w_hat sampled earlier), and `next` (one host descriptor, may be NULL) is sampled as
 * gws_sample_fwd(next, 1, fmt, step) would: next->w_hat and next->scale are written.  This is how a
 * forward pass that knows its layers hides the sampling of layer l+1 behind the GEMM of layer l
 * (the paper keeps sampling and matmul in separate kernels, Sec. 3.5; so does this, in one launch):
 * when the GEMM takes the 256-tile kernel and its last round of tiles leaves compute units idle,
 * that many extra workgroups of the same launch do the sampling there; otherwise the sampling kernel
 * is launched after the GEMM.  Same bytes either way; no state; next->w_hat must not overlap x, w
 * or y (GWS_ERR_ALIAS).                                                                        */
int gws_gemm_bf16_sample_next(const void* x, int64_t M, int64_t K, int64_t ldx,
                              const void* w, int64_t N, int64_t ldw, int w_is_nk,
                              void* y, int64_t ldy,
                              const gws_tensor* next, int fmt, uint64_t step, void* stream);

/* The same for a list of weights (host array of n_next <= 64 descriptors, sampled as gws_sample_fwd(next, n_next,
 * fmt, step) would): a forward pass that knows its layers can sample several coming weights under one GEMM whose
 * last round of tiles leaves many compute units idle, and none under a GEMM whose tiles fill the chip exactly.
 * As many weights as fit ride in the GEMM's launch, in the order given (at most four; riding several needs rows
 * a multiple of 32 and columns a multiple of 256); the rest are sampled by one launch after the GEMM.  Same
 * bytes either way.  n_next = 0 is gws_gemm_bf16.                                                        */
int gws_gemm_bf16_sample_next_n(const void* x, int64_t M, int64_t K, int64_t ldx,
                                const void* w, int64_t N, int64_t ldw, int w_is_nk,
                                void* y, int64_t ldy,
                                const gws_tensor* next, int n_next, int fmt, uint64_t step, void* stream);

/* The comparison systems of the paper's Sec. 4 behind the same interface: the same forward and
 * backward passes with R drawn from another noise basis.  The paper compares GaussWS with the same
 * pipeline on a BF16 U(-0.5, 0.5) basis (its "DiffQ" extension, Sec. 4 and Table 1) and, in the
 * forward unit benchmark (Sec. 4 "Overhead"), with the exact rounded normal round(N(0,1)/2) from a
 * Box-Muller transform ("bm"); it does not say how either is drawn from the random integers.  Here
 * both use the Philox call of the bit basis (same counter, same key) per group of 8 elements:
 *   GWS_BASIS_UNIFORM_BF16  element k (= j & 7) owns byte k % 4 of word k / 4;
 *                           R = (2 byte - 255) / 512, the 256 midpoints of a 1/256 grid on
 *                           (-0.5, 0.5): BF16 values, mean exactly 0, variance (1 - 2^-16) / 12.
 *                           R * s is not exact and is rounded to BF16 before the add:
 *                           w_hat = cast_fmt( bf16_rne( w + bf16_rne(R * s) ) ).
 *   GWS_BASIS_BOX_MULLER    the pair of elements (2d, 2d + 1) owns word d; u1 = (low half + 0.5) / 2^16,
 *                           u2 = (high half + 0.5) / 2^16, z = sqrt(-2 ln u1) (cos, sin)(2 pi u2) in
 *                           fp32 (one fixed sequence of operations), R = rint(z / 2) in {0, +-1, +-2}.
 *   GWS_BASIS_BITS          the method's own basis (Sec. 3.4): gws_sample_fwd / gws_sample_bwd.
 * Everything else (block maximum, scale, cast, Eq. 4 with this R) is as in gws_sample_fwd /
 * gws_sample_bwd; an unknown basis gives GWS_ERR_FORMAT.                                        */
typedef enum gws_basis { GWS_BASIS_BITS = 0, GWS_BASIS_UNIFORM_BF16 = 1, GWS_BASIS_BOX_MULLER = 2 } gws_basis;
int gws_sample_fwd_basis(const gws_tensor* t, int n, int basis, int fmt, uint64_t step, void* stream);
int gws_sample_bwd_basis(const gws_tensor* t, int n, int basis, uint64_t step, void* stream);

/* R of a comparison basis alone: out is device BF16 [rows x cols] (cols and col0 multiples of 8,
 * out 16-byte aligned), every R being a BF16 value (the Box-Muller basis keeps the sign on a zero).
 * basis is GWS_BASIS_UNIFORM_BF16 or GWS_BASIS_BOX_MULLER (the bit basis has gws_noise_packed).   */
int gws_noise_basis(void* out, int64_t rows, int64_t cols, int64_t row0, int64_t col0,
                    uint64_t seed, uint64_t step, int basis, void* stream);

/* The packed noise alone (paper Sec. 3.4: sign-magnitude, 4 bits per element,
 * 8 elements per 32-bit word): out is device u32 [rows x ceil(cols/8)], element
 * k of a group in bits 4k..4k+3, code = sign<<3 | |R|.  The training path never
 * materialises this tensor; the entry point exists to inspect R.                  */
int gws_noise_packed(void* out, int64_t rows, int64_t cols, int64_t row0, int64_t col0,
                     uint64_t seed, uint64_t step, void* stream);

/* Per-tensor seed from a user seed (paper Sec. 3.6: layers must draw independent
 * R).  Pure host function: low 64 bits of Philox4x32-10(counter = (id_lo, id_hi,
 * 0x47575331, 0), key = user seed).  The training loop passes step = index of the
 * gradient update, which replaces the paper's per-layer PRNG state.               */
uint64_t gws_derive_seed(uint64_t user_seed, uint64_t tensor_id);

const char* gws_status_string(int status);
int gws_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GWS_H */
