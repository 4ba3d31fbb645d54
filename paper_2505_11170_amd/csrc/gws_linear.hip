// BF16 MFMA GEMM for gfx950 with an optional GaussWS sampling stage in the
// weight-operand path: Y = X * w_hat (fused; paper Eq. 3 + cast applied to each
// 32x32 block of W on its way from global memory to LDS) or Y = X * W (plain
// twin, same tiling, used as the reference point for the fused overhead).
//
// Tiling.  Workgroup = 256 threads = 2x2 wavefronts, block tile 128 x 128 x 32;
// a wavefront owns 64 x 64 of the output as 2x2 v_mfma_f32_32x32x16_bf16 tiles.
// Both operands sit in LDS K-contiguous ([row][k], 80-byte row pitch), so every
// MFMA operand is one 16-byte LDS read per lane.  BK = 32 = b_l, hence one
// K-step of the weight tile holds whole 32x32 blocks: a wavefront loads exactly
// one block (two 16-byte groups per lane), reduces max|w| across its 64 lanes,
// samples in registers and writes w_hat to LDS.  Global loads for step k+1 are
// issued before the MFMAs of step k.
#include "gws_launch.h"

namespace gws {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDSP = BK + 8;  // LDS row pitch in elements (80 bytes)

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) v = max(v, (uint32_t)__shfl_xor((int)v, o));
  return v;
}

union Frag {
  uint4 u;
  bf16x8 v;
};

// W_NK: weight stored [N x K] (K contiguous) instead of [K x N].
template <bool FUSED, int FMT, bool W_NK>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmArgs g) {
  __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDSP];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * LDSP];

  const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const uint32_t n_tiles_n = (g.N + BN - 1) / BN;
  const uint32_t tile_m = blockIdx.x / n_tiles_n, tile_n = blockIdx.x % n_tiles_n;
  const uint32_t m0 = tile_m * BM, n0 = tile_n * BN;
  const uint32_t wm = wave >> 1, wn = wave & 1;

  // ---- global -> register staging -------------------------------------------
  // X tile: 128 rows x 32 k = 512 groups of 8; thread: row = tid/4 + 64 i, kgroup = tid%4
  const uint32_t a_kg = tid & 3;
  uint32_t a_row[2];
  const uint16_t* a_ptr[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    a_row[i] = (tid >> 2) + 64 * i;
    uint32_t r = m0 + a_row[i];
    r = r < g.M ? r : g.M - 1;  // clamp: rows past M are computed and discarded
    a_ptr[i] = g.x + (size_t)r * g.ldx + a_kg * 8;
  }
  // W tile: wavefront `wave` owns the 32x32 block at n-offset 32*wave of the tile.
  //   [N x K]: lane -> n = 32 wave + lane/4 + 16 i, k-group = lane%4
  //   [K x N]: lane -> k = lane/4 + 16 i,           n-group = 4 wave + lane%4
  const uint32_t b_q = lane & 3, b_r = lane >> 2;
  const uint32_t blk_n = n0 + 32 * wave;  // first n of this wave's block
  const bool blk_ok = blk_n < g.N;        // N is a multiple of 32: a block is whole or absent
  const uint16_t* b_ptr[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (W_NK) b_ptr[i] = g.w + (size_t)(blk_ok ? blk_n + b_r + 16 * i : 0) * g.ldw + b_q * 8;
    else b_ptr[i] = g.w + (size_t)(b_r + 16 * i) * g.ldw + (blk_ok ? blk_n + b_q * 8 : 0);
  }
  const uint32_t nbc = W_NK ? (g.K >> 5) : (g.N >> 5);  // blocks per storage row of b_t / scale

  u32x4 ra[2], rb[2];
  auto load_tiles = [&](uint32_t kt) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      ra[i] = *(const u32x4*)(a_ptr[i] + (size_t)kt * BK);
      if (W_NK) rb[i] = *(const u32x4*)(b_ptr[i] + (size_t)kt * BK);
      else rb[i] = *(const u32x4*)(b_ptr[i] + (size_t)kt * BK * g.ldw);
      if (!blk_ok) rb[i] = u32x4{0, 0, 0, 0};
    }
  };

  // Eq. 3 + cast on this wavefront's 32x32 block held in rb[0..1].
  auto sample_block = [&](uint32_t kt) {
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) m = absmax_pk(rb[i], m);
    m = max(m & 0xFFFFu, m >> 16);
    const uint32_t a16 = wave_max_u32(m);
    // storage coordinates of the block: (block row, block col) in the stored matrix
    const uint32_t brow = W_NK ? (blk_n >> 5) : kt;
    const uint32_t bcol = W_NK ? kt : (blk_n >> 5);
    const float btv = blk_ok ? g.bt[(size_t)brow * nbc + bcol] : 0.0f;
    BlockScale b = block_scale(a16, btv);
    if (FMT == 1) cast_constants<8, -6>(a16, b);
    if (FMT == 2) cast_constants<4, -2>(a16, b);
    const bool writer = blk_ok && tile_m == 0 && g.w_hat != nullptr;
    if (writer && lane == 0) g.scale[(size_t)brow * nbc + bcol] = b.s32;
    const bool hw = (FMT == 1) && b.hw_safe;  // uniform: the whole wavefront holds one block
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t srow = (W_NK ? blk_n : kt * 32) + b_r + 16 * i;        // storage row
      const uint32_t scol = (W_NK ? kt * 32 : blk_n) + b_q * 8;             // storage column
      const Noise n = group_noise(g.cg0 + (scol >> 3), g.row0 + srow, g.step_lo, g.step_hi,
                                  g.seed_lo, g.seed_hi);
      rb[i] = hw ? sample_group<FMT>(rb[i], n, b, true) : sample_group<FMT>(rb[i], n, b, false);
      if (writer) *(u32x4*)(g.w_hat + (size_t)srow * g.ldw + scol) = rb[i];
    }
  };

  auto store_lds = [&]() {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      *(u32x4*)(As + a_row[i] * LDSP + a_kg * 8) = ra[i];
      if (W_NK) {
        *(u32x4*)(Bs + (32 * wave + b_r + 16 * i) * LDSP + b_q * 8) = rb[i];
      } else {
        // transpose while storing: the lane holds 8 consecutive n at one k
        const uint32_t e[4] = {rb[i][0], rb[i][1], rb[i][2], rb[i][3]};
        const uint32_t k = b_r + 16 * i, nb = 32 * wave + b_q * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j)
          Bs[(nb + j) * LDSP + k] = (uint16_t)(e[j >> 1] >> ((j & 1) * 16));
      }
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  const uint32_t nk = g.K / BK;
  load_tiles(0);
  for (uint32_t kt = 0; kt < nk; ++kt) {
    if (FUSED) sample_block(kt);
    store_lds();
    __syncthreads();
    if (kt + 1 < nk) load_tiles(kt + 1);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      Frag fa[2], fb[2];
      const uint32_t koff = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i].u = *(const uint4*)(As + (64 * wm + 32 * i + (lane & 31)) * LDSP + koff);
        fb[i].u = *(const uint4*)(Bs + (64 * wn + 32 * i + (lane & 31)) * LDSP + koff);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[j].v, acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // ---- epilogue: fp32 -> BF16 (RNE), 32x32 accumulator layout:
  //      acc[e] is row 8*(e/4) + 4*(lane/32) + e%4, column lane%32 of the MFMA tile
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t col = n0 + 64 * wn + 32 * j + (lane & 31);
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const uint32_t row = m0 + 64 * wm + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (row < g.M && col < g.N) g.y[(size_t)row * g.ldy + col] = (uint16_t)bf16_rne_bits(acc[i][j][e]);
      }
    }
}

template <bool FUSED, int FMT>
static int launch_layout(const GemmArgs& g, int w_is_nk, dim3 grid, hipStream_t s) {
  if (w_is_nk) hipLaunchKernelGGL((gemm_kernel<FUSED, FMT, true>), grid, dim3(256), 0, s, g);
  else hipLaunchKernelGGL((gemm_kernel<FUSED, FMT, false>), grid, dim3(256), 0, s, g);
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

int launch_gemm(const GemmArgs& g, int w_is_nk, int fused, int fmt, hipStream_t stream) {
  const uint64_t tiles = (uint64_t)((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (tiles == 0) return GWS_OK;
  if (tiles >= 0x7FFFFFFFull) return GWS_ERR_SHAPE;
  const dim3 grid((uint32_t)tiles);
  if (!fused && gemm256_applicable(g)) return launch_gemm256(g, w_is_nk, stream);
  if (!fused) return launch_layout<false, 0>(g, w_is_nk, grid, stream);
  switch (fmt) {
    case GWS_FMT_BF16: return launch_layout<true, 0>(g, w_is_nk, grid, stream);
    case GWS_FMT_FP8_E4M3: return launch_layout<true, 1>(g, w_is_nk, grid, stream);
    case GWS_FMT_FP6_E3M2: return launch_layout<true, 2>(g, w_is_nk, grid, stream);
    default: return GWS_ERR_FORMAT;
  }
}

}  // namespace gws
