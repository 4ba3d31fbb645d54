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

// The way out of a wavefront's 128 x 128 part of dW (origin (p0, q0) in the weight): BF16 through the staging
// area, and with DBT the reduction of Eq. 4 over the groups as they pass.
template <bool DBT>
__device__ __forceinline__ void tn_write_half(const GemmArgs& g, const f32x4 (&a4)[4][8], int h, uint16_t* cs, uint32_t p0,
                                              uint32_t q0, uint32_t lane, float& part) {
  uint16_t* yw = g.y + (size_t)p0 * g.ldy + q0;
  if (!DBT) {
    epilogue_bf16_half(a4, h, cs, yw, g.ldy, lane, NoHook{});
    return;
  }
  const uint32_t nbc = g.N >> 5;
  // step `it` covers rows 4 it .. 4 it + 3 of the wavefront's part; lane = (row % 4, 16-byte column group)
  epilogue_bf16_half(a4, h, cs, yw, g.ldy, lane, [&](int it, uint32_t row, uint32_t c, const u32x4& v) {
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
__device__ __forceinline__ void gemm256_tn_tile(const GemmArgs& g, uint32_t L) {
  using namespace g256;
  uint32_t tile_m, tile_n;
  tile_of(L, g.M / TM, g.N / TN, tile_m, tile_n);
  const uint32_t m0 = tile_m * TM, n0 = tile_n * TN;
  gemm256_accumulate<true, true>(g.x, g.ldx, g.w, g.ldw, g.K / TK, m0, n0,
                                 [&](f32x4 (&acc)[8][8], uint16_t* cs, uint32_t wave, uint32_t lane) {
    const uint32_t p0 = m0 + 128 * (wave >> 1), q0 = n0 + 128 * (wave & 1);   // origin of the wavefront's part in dW
    float part = 0.0f;
    tn_write_half<DBT>(g, *reinterpret_cast<const f32x4 (*)[4][8]>(&acc[0]), 0, cs, p0, q0, lane, part);
    tn_write_half<DBT>(g, *reinterpret_cast<const f32x4 (*)[4][8]>(&acc[4]), 1, cs, p0, q0, lane, part);
  });
}

template <bool DBT>
__global__ __launch_bounds__(256, 1) void gemm256_tn_kernel(const GemmArgs g) {
  gemm256_tn_tile<DBT>(g, blockIdx.x);
}

// ---- the contraction split over several workgroups per tile ----
// A weight of few tiles (2048 x 2048: 64) leaves most compute units without work while each tile walks all tokens.
// Workgroup (tile L, part s) accumulates the tokens [kb, ke) of its part and leaves its accumulators in the
// workspace, as fp32 in register order (slab (s, L): 4 wavefronts x 64 accumulators x 64 lanes x 16 bytes, each
// store 1 KiB of consecutive memory); a second kernel adds a tile's parts in the order of s, rounds once to BF16 and
// goes out the same way as the one-kernel form (with the Eq. 4 reduction if asked for).  The result does not depend
// on timing: no atomics, no arrival order.
constexpr uint32_t kSlabFloats = 256 * 256;

__global__ __launch_bounds__(256, 1) void gemm256_tn_part_kernel(const GemmArgs g, float* __restrict__ ws, const uint32_t parts) {
  using namespace g256;
  const uint32_t tiles = (g.M / TM) * (g.N / TN);
  const uint32_t L = blockIdx.x % tiles, s = blockIdx.x / tiles;
  uint32_t tile_m, tile_n;
  tile_of(L, g.M / TM, g.N / TN, tile_m, tile_n);
  const uint32_t nk = g.K / TK;
  const uint32_t kb = (uint32_t)((uint64_t)nk * s / parts), ke = (uint32_t)((uint64_t)nk * (s + 1) / parts);
  float* slab = ws + ((size_t)s * tiles + L) * kSlabFloats;
  gemm256_accumulate<true, true>(g.x + (size_t)kb * TK * g.ldx, g.ldx, g.w + (size_t)kb * TK * g.ldw, g.ldw, ke - kb,
                                 tile_m * TM, tile_n * TN, [&](f32x4 (&acc)[8][8], uint16_t*, uint32_t wave, uint32_t lane) {
    f32x4* out = reinterpret_cast<f32x4*>(slab) + (size_t)wave * 64 * 64 + lane;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) out[(i * 8 + j) * 64] = acc[i][j];
  });
}

// One wavefront per workgroup, one half (64 x 128) of a wavefront's part of a tile each: eight workgroups per tile,
// so that a weight of 64 tiles spreads over the chip here too (the work is loads and little else).
template <bool DBT>
__global__ __launch_bounds__(64) void gemm256_tn_sum_kernel(const GemmArgs g, const float* __restrict__ ws, const uint32_t parts) {
  using namespace g256;
  __shared__ __attribute__((aligned(16))) uint16_t stage[64 * PC];
  const uint32_t tiles = (g.M / TM) * (g.N / TN);
  const uint32_t L = blockIdx.x >> 3, wave = (blockIdx.x >> 1) & 3, h = blockIdx.x & 1, lane = threadIdx.x;
  uint32_t tile_m, tile_n;
  tile_of(L, g.M / TM, g.N / TN, tile_m, tile_n);
  const uint32_t p0 = tile_m * TM + 128 * (wave >> 1), q0 = tile_n * TN + 128 * (wave & 1);
  f32x4 a4[4][8];
#pragma unroll
  for (int i2 = 0; i2 < 4; ++i2)
#pragma unroll
    for (int j = 0; j < 8; ++j) a4[i2][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  for (uint32_t s = 0; s < parts; ++s) {
    const f32x4* in = reinterpret_cast<const f32x4*>(ws + ((size_t)s * tiles + L) * kSlabFloats) + (size_t)wave * 64 * 64 + lane;
#pragma unroll
    for (int i2 = 0; i2 < 4; ++i2)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const f32x4 v = in[((4 * h + i2) * 8 + j) * 64];
#pragma unroll
        for (int e = 0; e < 4; ++e) a4[i2][j][e] = __fadd_rn(a4[i2][j][e], v[e]);
      }
  }
  float part = 0.0f;
  if (h == 0) tn_write_half<DBT>(g, a4, 0, stage, p0, q0, lane, part);
  else tn_write_half<DBT>(g, a4, 1, stage, p0, q0, lane, part);
}

bool gemm256_tn_applicable(const GemmArgs& g) {
  return g.M > 0 && g.N > 0 && g.K > 0 && g.M % g256::TM == 0 && g.N % g256::TN == 0 && g.K % g256::TK == 0 &&
         g.ldx < g256::kMaxLd && g.ldw < g256::kMaxLd;
}

int launch_gemm256_tn(const GemmArgs& g, bool with_dbt, hipStream_t stream) {
  const uint64_t tiles = (uint64_t)(g.M / g256::TM) * (g.N / g256::TN);
  if (tiles >= 0x7FFFFFFFull) return GWS_ERR_SHAPE;
  if (with_dbt) hipLaunchKernelGGL(gemm256_tn_kernel<true>, dim3((uint32_t)tiles), dim3(256), 0, stream, g);
  else hipLaunchKernelGGL(gemm256_tn_kernel<false>, dim3((uint32_t)tiles), dim3(256), 0, stream, g);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

size_t gemm256_tn_split_bytes(const GemmArgs& g, uint32_t parts) {
  return (size_t)parts * (g.M / g256::TM) * (g.N / g256::TN) * kSlabFloats * sizeof(float);
}

int launch_gemm256_tn_split(const GemmArgs& g, bool with_dbt, float* ws, uint32_t parts, hipStream_t stream) {
  const uint64_t tiles = (uint64_t)(g.M / g256::TM) * (g.N / g256::TN);
  if (parts < 2 || parts > g.K / g256::TK || tiles * parts >= 0x7FFFFFFFull || tiles * 8 >= 0x7FFFFFFFull) return GWS_ERR_SHAPE;
  hipLaunchKernelGGL(gemm256_tn_part_kernel, dim3((uint32_t)(tiles * parts)), dim3(256), 0, stream, g, ws, parts);
  if (hipGetLastError() != hipSuccess) return GWS_ERR_LAUNCH;
  if (with_dbt) hipLaunchKernelGGL(gemm256_tn_sum_kernel<true>, dim3((uint32_t)(tiles * 8)), dim3(64), 0, stream, g, (const float*)ws, parts);
  else hipLaunchKernelGGL(gemm256_tn_sum_kernel<false>, dim3((uint32_t)(tiles * 8)), dim3(64), 0, stream, g, (const float*)ws, parts);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

}  // namespace gws
