// Weight-gradient GEMM of the sampled-weight linear for gfx950, with the reduction of
// the paper's Eq. 4 in its epilogue:
//   C[P x Q] = A^T * B,  A [Mc x P], B [Mc x Q] row-major BF16 (contraction over the rows),
// i.e. dW = X^T dY for a weight stored [K x N] (A = X, B = dY) and dW = dY^T X for one
// stored [N x K] (A = dY, B = X); fp32 accumulation, one round-to-nearest-even to BF16.
// P, Q multiples of 256, Mc of 64.
//
// Same 256 x 256 x 64 tiling as the forward GEMM (2x2 wavefronts, each 4x4
// v_mfma_f32_32x32x16_bf16, two LDS stages).  Both operands arrive with the output index
// contiguous, so both tiles stay as loaded (544-byte pitch) and both MFMA operands are read
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
#include "gws_launch.h"
#include "gws_mfma.h"

namespace gws {

template <bool DBT>
__device__ __forceinline__ void gemm256_tn_tile(const GemmArgs& g, uint32_t L, uint16_t* lds) {
  using namespace g256;
  constexpr int STAGE = B_STAGE_KN;           // [TK][PB_KN] elements, for either operand
  uint16_t* const As = lds;                   // [2][STAGE]
  uint16_t* const Bs = lds + 2 * STAGE;       // [2][STAGE]

  const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const uint32_t wm = wave >> 1, wn = wave & 1;
  uint32_t tile_m, tile_n;
  tile_of(L, g.M / TM, g.N / TN, tile_m, tile_n);
  const uint32_t m0 = tile_m * TM, n0 = tile_n * TN;

  // ---- global -> register staging: thread = (contraction row tid/32, 8 output columns) ----
  const uint16_t* a_src = g.x + (size_t)(tid >> 5) * g.ldx + m0 + (tid & 31) * 8;   // + 8 rows per i
  const uint16_t* b_src = g.w + (size_t)(tid >> 5) * g.ldw + n0 + (tid & 31) * 8;
  u32x4 ra[8], rb[8];
  auto load_global = [&](uint32_t kt) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      ra[i] = *(const u32x4*)(a_src + (size_t)(kt * TK + 8 * i) * g.ldx);
      rb[i] = *(const u32x4*)(b_src + (size_t)(kt * TK + 8 * i) * g.ldw);
    }
  };
  auto store_lds = [&](uint32_t stage) {
    const uint32_t off = stage * STAGE + (tid >> 5) * PB_KN + (tid & 31) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      *(u32x4*)(As + off + 8 * i * PB_KN) = ra[i];
      *(u32x4*)(Bs + off + 8 * i * PB_KN) = rb[i];
    }
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // transposing read: group = lane / 16 -> output half (group & 1), k half (group >> 1);
  // lane i of a group points at contraction row k0 + i/4, output columns o0 + 4 (i%4)
  const uint32_t li = lane & 15, grp = lane >> 4;
  const uint32_t rd = ((grp >> 1) * 8 + (li >> 2)) * PB_KN + (grp & 1) * 16 + (li & 3) * 4;
  const uint32_t a_rd = rd + 128 * wm, b_rd = rd + 128 * wn;

  const uint32_t nk = g.K / TK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (uint32_t kt = 0; kt < nk; ++kt) {
    const uint32_t st = kt & 1;
    if (kt + 1 < nk) load_global(kt + 1);
    const uint16_t* a_s = As + st * STAGE;
    const uint16_t* b_s = Bs + st * STAGE;
#pragma unroll 2
    for (int ks = 0; ks < TK / 16; ++ks) {
      Frag8 fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint16_t* p = a_s + a_rd + (ks * 16) * PB_KN + 32 * i;
        fa[i].h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)p);
        fa[i].h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p + 4 * PB_KN));
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint16_t* p = b_s + b_rd + (ks * 16) * PB_KN + 32 * j;
        fb[j].h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)p);
        fb[j].h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p + 4 * PB_KN));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[j].v, acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_lds(st ^ 1);
    __syncthreads();
  }

  // ---- epilogue: fp32 -> BF16 (RNE) into LDS, then 16-byte rows to global ----
  // acc[i][j][e]: row 32 i + 8 (e/4) + 4 (lane/32) + e%4, column 32 j + lane%32 of the wave tile
  uint16_t* cs = lds + wave * (128 * PC);
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const uint32_t row = 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        cs[row * PC + 32 * j + (lane & 31)] = (uint16_t)bf16_rne_bits(acc[i][j][e]);
      }
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wavefront's LDS writes have landed
  __builtin_amdgcn_wave_barrier();
  const uint32_t p0 = m0 + 128 * wm, q0 = n0 + 128 * wn;      // origin of the wave tile in dW
  uint16_t* y = g.y + (size_t)p0 * g.ldy + q0;
  // lane = (row in a group of 4, 16-byte column group): 16 lanes x 8 columns = 128 columns
  const uint32_t lr = lane >> 4, c = (lane & 15) * 8;
  const uint32_t nbc = g.N >> 5;
  float part = 0.0f;
#pragma unroll 4
  for (int it = 0; it < 32; ++it) {
    const uint32_t row = it * 4 + lr;
    const u32x4 v = *(const u32x4*)(cs + row * PC + c);
    *(u32x4*)(y + (size_t)row * g.ldy + c) = v;
    if (DBT) {
      const Noise n = group_noise(g.cg0 + ((q0 + c) >> 3), g.row0 + p0 + row, g.step_lo, g.step_hi, g.seed_lo, g.seed_hi);
      part = dot_group_2r(v, n, part);
      if ((it & 7) == 7) {
        // rows 32 b .. 32 b + 31 are done: the block's 16 lanes (4 column groups x 4 row lanes) reduce
        float s = part;
        s += __uint_as_float(dpp_u32<0xB1>(__float_as_uint(s)));   // lane ^ 1
        s += __uint_as_float(dpp_u32<0x4E>(__float_as_uint(s)));   // lane ^ 2
        s += __uint_as_float((uint32_t)__builtin_amdgcn_ds_swizzle((int)__float_as_uint(s), 0x401F));  // lane ^ 16
        s += __shfl_xor(s, 32);
        if ((lane & 3) == 0 && lr == 0) {
          const size_t blk = (size_t)((p0 >> 5) + (it >> 3)) * nbc + (q0 >> 5) + ((lane & 15) >> 2);
          const float neg_ln2 = __uint_as_float(0xBF317218u);  // -ln 2
          g.dbt[blk] = (neg_ln2 * g.scale[blk]) * (s * 0.5f);
        }
        part = 0.0f;
      }
    }
  }
}

template <bool DBT>
__global__ __launch_bounds__(256, 1) void gemm256_tn_kernel(const GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  gemm256_tn_tile<DBT>(g, blockIdx.x, lds);
}

bool gemm256_tn_applicable(const GemmArgs& g) {
  return g.M > 0 && g.N > 0 && g.K > 0 && g.M % g256::TM == 0 && g.N % g256::TN == 0 && g.K % g256::TK == 0;
}

int launch_gemm256_tn(const GemmArgs& g, bool with_dbt, hipStream_t stream) {
  const uint64_t tiles = (uint64_t)(g.M / g256::TM) * (g.N / g256::TN);
  if (tiles >= 0x7FFFFFFFull) return GWS_ERR_SHAPE;
  constexpr size_t lds = g256::lds_bytes_tn();
  static_assert(lds >= (size_t)4 * 128 * g256::PC * 2, "the epilogue staging fits the operand stages");
  if (with_dbt) {
    static const bool ok = hipFuncSetAttribute((const void*)gemm256_tn_kernel<true>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
    if (!ok) return GWS_ERR_LAUNCH;
    hipLaunchKernelGGL(gemm256_tn_kernel<true>, dim3((uint32_t)tiles), dim3(256), lds, stream, g);
  } else {
    static const bool ok = hipFuncSetAttribute((const void*)gemm256_tn_kernel<false>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
    if (!ok) return GWS_ERR_LAUNCH;
    hipLaunchKernelGGL(gemm256_tn_kernel<false>, dim3((uint32_t)tiles), dim3(256), lds, stream, g);
  }
  return hipGetLastError() == hipSuccess ? GWS_OK : GWS_ERR_LAUNCH;
}

}  // namespace gws
