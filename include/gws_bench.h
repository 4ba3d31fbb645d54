/*
 * libgws -- measurement aids.  Not part of the method: these calls move the bytes of the
 * GaussWS forward and backward passes (paper Eq. 3, Eq. 4) with the launch shape, loads and
 * stores of gws_sample_fwd / gws_sample_bwd and none of their arithmetic, so that a benchmark
 * can put the rate of the sampling kernels next to the rate the memory system allows for the
 * same access pattern.  Same conventions as gws.h: device pointers owned by the caller, host
 * descriptor array read before the call returns, asynchronous on the given stream, gws_status
 * returned, nothing launched on error.
 */
#ifndef GWS_BENCH_H
#define GWS_BENCH_H

#include "gws.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Copies w to w_hat for n tensors with the launch shape, loads and stores of gws_sample_fwd.
 * Its rate is the ceiling the memory system sets for that access pattern, against which the
 * forward pass is read.  Uses fields w, w_hat, rows, cols, ld.                              */
int gws_copy_tiles(const gws_tensor* t, int n, void* stream);

/* Step one of Eq. 3 alone: writes max_{b_l}|w| (exact, as fp32) of every 32x32 block into
 * `scale`, for n tensors, with the launch shape and loads of gws_sample_bwd.  It reads
 * each element once and writes 4 bytes per block, so its rate is the ceiling the memory
 * system sets for the backward pass.  Uses fields w, scale, rows, cols, ld.                 */
int gws_block_absmax(const gws_tensor* t, int n, void* stream);

/* gws_sample_bwd with the launch shape chosen by the caller, to measure the choices the library makes:
 *   variant  -1 = the library's choice; 0 = the kernel for any shape; 1 = the whole-tile kernel (used only
 *            where every tensor of a launch has rows % 32 == 0, cols % 256 == 0 and an aliased dL/dw)
 *   per_x    column tiles (256 columns) one workgroup walks; 0 = the library's choice
 * Same results as gws_sample_bwd whatever the choice.                                                  */
int gws_sample_bwd_tuned(const gws_tensor* t, int n, uint64_t step, int variant, int per_x, void* stream);

/* The same for gws_sample_fwd: variant -1 / 0 / 1 (whole-tile kernel), per_x as above.               */
int gws_sample_fwd_tuned(const gws_tensor* t, int n, int fmt, uint64_t step, int variant, int per_x, void* stream);

/* gws_gemm_bf16_sample_next with the riding forced: the GEMM (none at all if M == 0) is followed in the same
 * grid by `extra_workgroups` (1 .. 4096) workgroups that sample `next` (rows a multiple of 32, columns of 64),
 * whatever the library's own estimate of whether the sampling fits beside the GEMM's last round says.
 * rider: 0 = the riding loop for any such weight, 1 = the loop for weights of whole 32 x 256 tiles (falls back
 * to 0 for other weights).  Same bytes as gws_gemm_bf16_sample_next.                                        */
int gws_gemm_bf16_ride_probe(const void* x, int64_t M, int64_t K, int64_t ldx, const void* w, int64_t N, int64_t ldw,
                             int w_is_nk, void* y, int64_t ldy, const gws_tensor* next, int fmt, uint64_t step,
                             int extra_workgroups, int rider, void* stream);

/* How many of the weights next[0 .. n_next) gws_gemm_bf16_sample_next_n would let ride in the launch of an
 * M x K x N GEMM on the current device (a prefix of the list); host function, launches nothing.            */
int gws_ride_plan(int64_t M, int64_t K, int64_t N, const gws_tensor* next, int n_next);

#ifdef __cplusplus
}
#endif
#endif /* GWS_BENCH_H */
