// Weight-gradient GEMM of the sampled-weight linear for gfx950, with the reduction of
// the paper's Eq. 4 in its epilogue:
//   C[P x Q] = A^T * B,  A [Mc x P], B [Mc x Q] row-major BF16 (contraction over the rows),
// i.e. dW = X^T dY for a weight stored [K x N] (A = X, B = dY) and dW = dY^T X for one
// stored [N x K] (A = dY, B = X); fp32 accumulation, one round-to-nearest-even to BF16.
// P, Q multiples of 256, Mc of 64.
//
// Same 256 x 256 x 64 tile as the forward GEMM (gws_gemm256_core.h).  Both operands arrive with
// the output index contiguous, so both tiles stay as loaded and both MFMA operands are read
// with the transposing LDS load (ds_read_b64_tr_b16).
//
// Epilogue: the BF16 tile is staged in LDS and written 16 bytes per lane; a 16-byte group is
// 8 consecutive elements of a row of dW, exactly what one Philox call covers, and the 32x32
// blocks of the weight coincide with 32-row x 32-column pieces of the wavefront's 128 x 128
// tile.  On the way out each lane regenerates R for its groups (same seed, step and
// coordinates as the forward pass), accumulates dW .* 2R with v_dot2c_f32_bf16 over the 8
// groups it owns of a block, the 16 lanes of the block reduce, and one lane writes
//   dL/db_t = -ln2 * s32 * sum(dW .* R)
// computed on the rounded BF16 dW, as gws_sample_bwd would from the same bytes.
#include "gws_gemm256_core.h"
#include "gws_launch.h"

namespace gws {

template <bool DBT>
__device__ __forceinline__ void gemm256_tn_tile(const GemmArgs& g, uint32_t L) {
  using namespace g256;
  uint32_t tile_m, tile_n;
  tile_of(L, g.M / TM, g.N / TN, tile_m, tile_n);
  const uint32_t m0 = tile_m * TM, n0 = tile_n * TN;
  if (!DBT) {
    gemm256_core<true, true>(g.x, g.ldx, g.w, g.ldw, g.y, g.ldy, g.K / TK, m0, n0, NoHook{});
    return;
  }
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t p0 = m0 + 128 * (wave >> 1), q0 = n0 + 128 * (wave & 1);   // origin of the wavefront tile in dW
  const uint32_t nbc = g.N >> 5;
  float part = 0.0f;
  // step `it` covers rows 4 it .. 4 it + 3 of the wavefront tile; lane = (row % 4, 16-byte column group)
  gemm256_core<true, true>(g.x, g.ldx, g.w, g.ldw, g.y, g.ldy, g.K / TK, m0, n0,
                           [&](int it, uint32_t row, uint32_t c, const u32x4& v) {
    const Noise n = group_noise(g.cg0 + ((q0 + c) >> 3), g.row0 + p0 + row, g.step_lo, g.step_hi, g.seed_lo, g.seed_hi);
    part = dot_group_2r(v, n, part);
    if ((it & 7) == 7) {
      // rows 32 b .. 32 b + 31 are done: the block's 16 lanes (4 column groups x 4 row lanes) reduce
      float s = part;
      s += __uint_as_float(dpp_u32<0xB1>(__float_as_uint(s)));   // lane ^ 1
      s += __uint_as_float(dpp_u32<0x4E>(__float_as_uint(s)));   // lane ^ 2
      s += __uint_as_float((uint32_t)__builtin_amdgcn_ds_swizzle((int)__float_as_uint(s), 0x401F));  // lane ^ 16
      s += __shfl_xor(s, 32);
      if ((lane & 3) == 0 && (lane >> 4) == 0) {
        const size_t blk = (size_t)((p0 >> 5) + (it >> 3)) * nbc + (q0 >> 5) + ((lane & 15) >> 2);
        const float neg_ln2 = __uint_as_float(0xBF317218u);  // -ln 2
        g.dbt[blk] = (neg_ln2 * g.scale[blk]) * (s * 0.5f);
      }
      part = 0.0f;
    }
  });
}

template <bool DBT>
__global__ __launch_bounds__(256, 1) void gemm256_tn_kernel(const GemmArgs g) {
  gemm256_tn_tile<DBT>(g, blockIdx.x);
}

bool gemm256_tn_applicable(const GemmArgs& g) {
  return g.M > 0 && g.N > 0 && g.K > 0 && g.M % g256::TM == 0 && g.N % g256::TN == 0 && g.K % g256::TK == 0;
}

int launch_gemm256_tn(const GemmArgs& g, bool with_dbt, hipStream_t stream) {
  const uint64_t tiles = (uint64_t)(g.M / g256::TM) * (g.N / g256::TN);
  if (tiles >= 0x7FFFFFFFull) return GWS_ERR_SHAPE;
  if (with_dbt) hipLaunchKernelGGL(gemm256_tn_kernel<true>, dim3((uint32_t)tiles), dim3(256), 0, stream, g);
  else hipLaunchKernelGGL(gemm256_tn_kernel<false>, dim3((uint32_t)tiles), dim3(256), 0, stream, g);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

}  // namespace gws
