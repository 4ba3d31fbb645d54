// One 256 x 256 output tile of a BF16 GEMM on gfx950, shared by the large-tile kernels
// (internal to csrc/).
//
// Workgroup = 256 threads = 2x2 wavefronts, K-steps of 64; a wavefront owns 128 x 128 of the
// output as 8x8 v_mfma_f32_16x16x32_bf16 tiles (256 accumulator registers per lane, one
// wavefront per SIMD).  The GEMM runs against the card's power limit, and on random operands
// the 16x16x32 MFMA takes less energy per flop than the 32x32x16 one (a loop of MFMAs alone is
// 15 % faster with it, with the LDS reads and loads of this kernel 11 %).
//
// Operand tiles travel global -> LDS directly (global_load_lds_dwordx4, 16 bytes per lane, no
// staging registers), the A operand into a ring of two stages, the B operand (the weight) into a
// ring of three: 5 x 32 KiB, all of the 160 KiB of LDS.  In a training step the activations were
// written just before and come from the caches, the weights come from HBM; the third B stage
// doubles the time a weight load may take (about one K-step with two stages).  Such a load
// writes its 64 lanes to 1 KiB of consecutive LDS, so the layout is unpadded and bank conflicts
// are avoided by choosing which 16-byte chunk of the tile each lane fetches (an XOR swizzle of
// the chunk index):
//   operand stored contraction-contiguous (X; a weight stored [N x K]): tile = 256 rows of
//     128 bytes; chunk c of row r sits in slot c ^ ((r / 2) % 8), so that any 16 rows a
//     ds_read_b128 serves together (two rows share 64 banks) hit 16 different bank groups; one
//     such read per MFMA operand;
//   operand stored output-contiguous (a weight stored [K x N]; both operands of the
//     weight-gradient GEMM): tile = 64 k-rows of 512 bytes; chunk c of row k sits in slot
//     c ^ 4 (k % 4) ^ 2 (k / 8 % 2) (the 32 lanes one such read serves together take four rows
//     k % 4 of two row groups k / 8, and every row starts at bank 0); read with the transposing LDS load
//     (ds_read_b64_tr_b16: within 16 lanes,
//     lanes 4j..4j+3 point at 16 consecutive outputs of row k0+j and lane i receives the four k
//     of output o0+i; the four 16-lane groups take the four 8-deep parts of the MFMA's k = 32),
//     two per MFMA operand.
// The stage arrays are separate LDS variables and the direct loads are issued from assembly
// statements: the compiler orders every LDS read it cannot tell apart after every direct load
// it knows of (s_waitcnt vmcnt(0)), which would expose the load latency in every K-step and
// defeat the ring.  The waits for the loads are the explicit ones in front of the barriers
// (loads complete in order: "all but the last 8" leaves the youngest B stage in flight).
//
// With one wavefront per SIMD nothing else hides latency, and left to itself the scheduler
// puts each LDS read right before its use and the 16 loads of a K-step in one burst, both of
// which stall the MFMA pipe.  The order of the main loop is therefore written out and pinned
// (a scheduling barrier after every step): the 64 MFMAs of a 32-deep slice are interleaved
// with the LDS reads of the next slice (into the other fragment buffer), at most one behind an
// MFMA, and, in the second slice of a K-step, with its 16 loads, one behind every fourth MFMA.
// The single barrier of a K-step sits between its two slices: in front of it every wavefront
// waits for its reads of the stages (so they can be refilled, A for the step after next, B for
// the one after that) and for its share of the next step's stages, whose first fragments are
// then fetched under the second slice's MFMAs.
#pragma once

#include "gws_device.h"
#include "gws_launch.h"

namespace gws {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define GWS_LDS __attribute__((address_space(3)))

namespace g256 {
constexpr int TM = 256, TN = 256, TK = 64;
constexpr int STAGE = 256 * 64;   // elements of one operand tile (32 KiB), either layout
constexpr int PC = 128 + 8;       // epilogue pitch of a wavefront's staging rows (elements)
constexpr uint32_t kMaxLd = 1u << 28;   // leading dimensions (elements) the 32-bit lane offsets of the loads reach: 7 rows x 2 bytes
static_assert(64 * PC <= STAGE, "half a wavefront tile is staged in one stage array");
}  // namespace g256

union Frag8 {
  u32x4 u;
  bf16x8 v;
  i16x4 h[2];
};

// XCD-aware tile numbering: launch-order number L -> (tile_m, tile_n) of an mt x nt grid of
// tiles.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2; XCD x gets
// a contiguous range of an order that walks 8 m-tiles down before moving one n-tile right,
// so the 32 workgroups running together on an XCD form an 8 x 4 patch sharing 8 + 4 panels.
__device__ __forceinline__ void tile_of(uint32_t L, uint32_t mt, uint32_t nt, uint32_t& tile_m, uint32_t& tile_n) {
  const uint32_t total = mt * nt;
  const uint32_t per = total / 8, rem = total % 8, x = L % 8, j = L / 8;
  L = x * per + (x < rem ? x : rem) + j;            // XCD x owns `per` tiles (+1 for the first `rem`)
  const uint32_t band_sz = 8 * nt;                   // tiles in a band of 8 m-tiles
  const uint32_t band = L / band_sz, r = L % band_sz;
  const uint32_t mrows = (band * 8 + 8 <= mt) ? 8 : (mt - band * 8);  // last band may be short
  tile_n = r / mrows;
  tile_m = band * 8 + r % mrows;
}

// Half h (rows 64 h .. 64 h + 63) of a wavefront's 128 x 128 part of the result on its way out: fp32 -> BF16 (RNE)
// into the wavefront's staging area `cs` (64 rows of pitch PC; 8 bytes per lane: its four consecutive columns),
// then 16-byte groups to yw[(64 h + row) * ldy + col], each also handed to hook(it, row, col, v) with it = 16 h + the
// 4-row step, row and col relative to the wavefront's part, lane = (row % 4, col / 8).
// a4[i2][j][e]: row 64 h + 16 i2 + lane % 16, column 16 j + 4 (lane / 16) + e.
template <class Hook>
__device__ __forceinline__ void epilogue_bf16_half(const f32x4 (&a4)[4][8], int h, uint16_t* cs, uint16_t* yw, uint32_t ldy,
                                                   uint32_t lane, Hook&& hook) {
  using namespace g256;
  const uint32_t li = lane & 15, grp = lane >> 4, lr = lane >> 4, c = (lane & 15) * 8;
#pragma unroll
  for (int i2 = 0; i2 < 4; ++i2)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const f32x4 v = a4[i2][j];
      u32x2 pk;
      pk[0] = pack_bf16_rne(v[0], v[1]);
      pk[1] = pack_bf16_rne(v[2], v[3]);
      *(u32x2*)(cs + (16 * i2 + li) * PC + 16 * j + 4 * grp) = pk;
    }
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wavefront's LDS writes have landed
  __builtin_amdgcn_wave_barrier();
#pragma unroll 4
  for (int it = 0; it < 16; ++it) {
    const uint32_t row = it * 4 + lr;
    const u32x4 v = *(const u32x4*)(cs + row * PC + c);
    *(u32x4*)(yw + (size_t)(64 * h + row) * ldy + c) = v;
    hook(16 * h + it, 64 * h + row, c, v);
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);  // the reads are done before the staging area is written again
  __builtin_amdgcn_wave_barrier();
}

// The accumulators of the C tile at (m0, n0) = sum over nk K-steps of A-tile * B-tile, handed to
// finish(acc, cs, wave, lane) when the last MFMA has retired:
//   A_OC = false: a[(m0 + r) * lda + k]   (contraction-contiguous)   true: a[k * lda + m0 + r]
//   B_OC = false: b[(n0 + c) * ldb + k]                               true: b[k * ldb + n0 + c]
//   acc[i][j][e]: row 16 i + lane % 16, column 16 j + 4 (lane / 16) + e of the wavefront's 128 x 128 part, which
//   starts at row 128 (wave / 2), column 128 (wave % 2) of the tile; cs: 64 x PC elements of LDS that are the
//   wavefront's own from here on (a stage array nobody reads any more).
// Requires nk >= 1 and all 256 threads; ends with every wavefront past its last LDS access
// except its own staging area (callers that loop over tiles put a barrier between tiles).
template <bool A_OC, bool B_OC, class Finish>
__device__ __forceinline__ void gemm256_accumulate(const uint16_t* __restrict__ a, uint32_t lda,
                                                   const uint16_t* __restrict__ b, uint32_t ldb, uint32_t nk, uint32_t m0,
                                                   uint32_t n0, Finish&& finish) {
  using namespace g256;
  __shared__ __attribute__((aligned(16))) uint16_t A0[STAGE];
  __shared__ __attribute__((aligned(16))) uint16_t A1[STAGE];
  __shared__ __attribute__((aligned(16))) uint16_t B0[STAGE];
  __shared__ __attribute__((aligned(16))) uint16_t B1[STAGE];
  __shared__ __attribute__((aligned(16))) uint16_t B2[STAGE];

  const uint32_t tid = threadIdx.x, lane = tid & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t wm = wave >> 1, wn = wave & 1;

  // ---- loads: wave-uniform base + per-lane byte offset; instruction q (0..7) of a wavefront fills
  // 1 KiB at (wave * 8 + q) * 1 KiB of the stage ----
  struct Src {
    const GWS_GLOBAL char* base;
    uint32_t voff[4];   // per-lane byte offset; which one an instruction q uses: vsel(oc, q)
    uint32_t ld;
  };
  auto make_src = [&](bool oc, const uint16_t* p, uint32_t ld, uint32_t o0) {
    Src s;
    s.ld = ld;
    if (!oc) {  // rows 64 wave + 8 q + lane/8; slot lane%8 holds chunk slot ^ ((row / 2) % 8) = slot ^ (4 (q%2) + lane/16)
      s.base = (const GWS_GLOBAL char*)(p + (size_t)(o0 + 64 * wave) * ld);
      s.voff[0] = s.voff[2] = ((lane >> 3) * ld + (((lane & 7) ^ (0 + (lane >> 4))) * 8)) * 2;
      s.voff[1] = s.voff[3] = ((lane >> 3) * ld + (((lane & 7) ^ (4 + (lane >> 4))) * 8)) * 2;
    } else {    // k-rows k = 16 wave + 2 q + lane/32; slot lane%32 holds chunk slot ^ 4 (k % 4) ^ 2 (k/8 % 2),
                // k % 4 = 2 (q%2) + lane/32, k/8 % 2 = q/4
      const uint32_t kb = lane >> 5;
      s.base = (const GWS_GLOBAL char*)(p + (size_t)(16 * wave) * ld + o0);
#pragma unroll
      for (int v = 0; v < 4; ++v)
        s.voff[v] = (kb * ld + (((lane & 31) ^ ((2 * (v & 1) + kb) << 2) ^ ((v >> 1) << 1)) * 8)) * 2;
    }
    return s;
  };
  const Src sa = make_src(A_OC, a, lda, m0), sb = make_src(B_OC, b, ldb, n0);
  auto load1 = [&](bool oc, const Src& s, uint16_t* stage, uint32_t kt, int q) {
    const size_t uni = oc ? (size_t)(kt * TK + 2 * q) * s.ld : (size_t)(8 * q) * s.ld + kt * TK;   // elements
    // issued from an assembly statement: the compiler would order every later read of the stage arrays after all
    // direct loads it knows of (vmcnt(0)), and the ring keeps loads in flight across the barrier on purpose; the
    // waits for these loads are the explicit ones in front of the barriers
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(GWS_LDS void*)(stage + (wave * 8 + q) * 512);
    // (m0, the LDS address register of such a load, is reserved to the compiler, which warns when told that it is
    // overwritten; it has to be told)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(s.voff[oc ? (q & 1) + 2 * ((q >> 2) & 1) : (q & 1)]), "s"(s.base + uni * 2), "s"(lds_addr) : "m0", "memory");
#pragma clang diagnostic pop
  };
  // load n (0..15) of a K-step: even n -> A, odd n -> B
  auto load_n = [&](uint16_t* As, uint16_t* Bs, uint32_t kt, int n) {
    if (!(n & 1)) load1(A_OC, sa, As, kt, n >> 1);
    else load1(B_OC, sb, Bs, kt, n >> 1);
  };

  // ---- fragment reads: per-lane element offsets into a stage ----
  // A fragment of the 16x16x32 MFMA is 16 outputs x 32 k: lane l holds output l % 16, k = 8 (l / 16) .. + 7.
  const uint32_t li = lane & 15, grp = lane >> 4, sw = (li >> 2) & 3;
  uint32_t a_off[4], b_off[4];   // contraction-contiguous: [ks] (2 used); output-contiguous: [fragment / 2]
  auto make_off = [&](bool oc, uint32_t w, uint32_t (&off)[4]) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (!oc) off[t] = (128 * w + li) * 64 + (((4 * (t & 1) + grp) ^ ((lane >> 1) & 7)) * 8);
      else off[t] = (8 * grp + (li >> 2)) * 256 + (16 * w + 4 * (t ^ sw) + ((li >> 1) & 1)) * 8 + (li & 1) * 4 + (grp & 1) * 16;
    }
  };
  make_off(A_OC, wm, a_off);
  make_off(B_OC, wn, b_off);
  // read `half` of fragment f (0..7) of slice ks (0, 1) from a stage
  auto read_frag = [&](bool oc, const uint32_t (&off)[4], Frag8& fr, const uint16_t* stage, int ks, int f, int half) {
    if (!oc) {
      fr.u = *(const u32x4*)(stage + off[ks] + f * 16 * 64);
    } else {
      const uint16_t* p = stage + (off[f >> 1] ^ ((f & 1) * 16)) + ks * 32 * 256 + half * 4 * 256;
      fr.h[half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GWS_LDS i16x4*)p);
    }
  };
  constexpr int RA = A_OC ? 2 : 1, RB = B_OC ? 2 : 1;   // LDS reads per fragment
  constexpr int NR = 8 * RA + 8 * RB;                   // reads per slice: 16, 24 or 32
  constexpr int RSTRIDE = 2;                            // one read every second MFMA: the last one is issued well before
                                                        // the wait in front of the barrier (measured: 2-3 % on the
                                                        // 16-read form against a read every fourth MFMA)
  static_assert(RSTRIDE * NR <= 64, "the reads of a slice fit behind its MFMAs");
  Frag8 fa[2][8], fb[2][8];
  // read n (0..NR-1) of slice (stage, ks) into fragment buffer `buf`, in the order the MFMAs need them:
  // A fragment 0, B fragments 0..7, A fragments 1..7
  auto read_n = [&](int buf, const uint16_t* As, const uint16_t* Bs, int ks, int n) {
    if (n < RA) {
      read_frag(A_OC, a_off, fa[buf][0], As, ks, 0, n);
    } else if (n < RA + 8 * RB) {
      const int m = n - RA;
      read_frag(B_OC, b_off, fb[buf][m / RB], Bs, ks, m / RB, m % RB);
    } else {
      const int m = n - RA - 8 * RB;
      read_frag(A_OC, a_off, fa[buf][1 + m / RA], As, ks, 1 + m / RA, m % RA);
    }
  };

  // acc[i][j]: the MFMA takes the B fragment as its first operand, so that a lane ends up with four
  // consecutive columns of one row: row 16 i + lane % 16, columns 16 j + 4 (lane / 16) .. + 3 of the wavefront tile
  f32x4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.0f;
  auto mfma_n = [&](int buf, int n) {
    // the B fragments go up and down again: at a change of the A fragment the other operand stays
    const int i = n >> 3, j = (i & 1) ? 7 - (n & 7) : (n & 7);
    // written as assembly so that the accumulator is one register tuple, tied in and out: with the builtin the
    // compiler moves accumulators between registers at every turn of the loop
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fb[buf][j].u), "v"(fa[buf][i].u));
  };

  // One K-step on the stages (Ac, Bc).  The A operand lives in a ring of two stages, the B operand (the weight,
  // which comes from HBM where the activations come from the caches) in a ring of three: K-step k computes on
  // A[k % 2], B[k % 3]; its second slice requests A of K-step k + 2 (`ka`) into Ac and B of K-step k + 3 (`kb`) into Bc,
  // the A loads first.  Loads complete in order, so "all but the last 8" at the barrier means: A and B of the next
  // K-step have landed, the B loads of the K-step after it may still be in flight.
  auto kstep = [&](uint16_t* Ac, uint16_t* Bc, uint16_t* An, uint16_t* Bn, uint32_t ka, uint32_t kb) {
#pragma unroll
    for (int n = 0; n < 64; ++n) {
      mfma_n(0, n);
      __builtin_amdgcn_sched_barrier(0);
      if (n % RSTRIDE == 0 && n / RSTRIDE < NR) {
        read_n(1, Ac, Bc, 1, n / RSTRIDE);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int n = 0; n < 64; ++n) {
      mfma_n(1, n);
      __builtin_amdgcn_sched_barrier(0);
      if (n % 4 == 1) {
        const int idx = n / 4;
        if (idx < 8) load1(A_OC, sa, Ac, ka, idx);
        else load1(B_OC, sb, Bc, kb, idx - 8);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (n % RSTRIDE == 0 && n / RSTRIDE < NR) {
        read_n(0, An, Bn, 0, n / RSTRIDE);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  // Past the last K-step the loads refetch that step into stages nobody reads any more and
  // the fragment reads go unused: no branches in the loop body.
  const uint32_t last = nk - 1;
  auto cl = [&](uint32_t k) { return k < last ? k : last; };
  // everything the rings hold is requested at once (one memory round trip in front of the first MFMA)
#pragma unroll
  for (int n = 0; n < 16; ++n) load_n(A0, B0, 0, n);
#pragma unroll
  for (int q = 0; q < 8; ++q) load1(A_OC, sa, A1, cl(1), q);
#pragma unroll
  for (int q = 0; q < 8; ++q) load1(B_OC, sb, B1, cl(1), q);
#pragma unroll
  for (int q = 0; q < 8; ++q) load1(B_OC, sb, B2, cl(2), q);
  asm volatile("s_waitcnt vmcnt(24)\n\ts_barrier" ::: "memory");   // the first stages have landed
#pragma unroll
  for (int n = 0; n < NR; ++n) read_n(0, A0, B0, 0, n);
  // the compiler does not know that the assembly statements are MFMAs: keep the zeroing of the accumulators
  // (vector writes) the required wait states away from the first of them
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_nop 3");
  __builtin_amdgcn_sched_barrier(0);
  uint32_t kt = 0;
  for (; kt + 6 <= nk; kt += 6) {
    kstep(A0, B0, A1, B1, cl(kt + 2), cl(kt + 3));
    kstep(A1, B1, A0, B2, cl(kt + 3), cl(kt + 4));
    kstep(A0, B2, A1, B0, cl(kt + 4), cl(kt + 5));
    kstep(A1, B0, A0, B1, cl(kt + 5), cl(kt + 6));
    kstep(A0, B1, A1, B2, cl(kt + 6), cl(kt + 7));
    kstep(A1, B2, A0, B0, cl(kt + 7), cl(kt + 8));
  }
  const uint32_t rem = nk - kt;
  if (rem > 0) kstep(A0, B0, A1, B1, cl(kt + 2), cl(kt + 3));
  if (rem > 1) kstep(A1, B1, A0, B2, cl(kt + 3), cl(kt + 4));
  if (rem > 2) kstep(A0, B2, A1, B0, cl(kt + 4), cl(kt + 5));
  if (rem > 3) kstep(A1, B0, A0, B1, cl(kt + 5), cl(kt + 6));
  if (rem > 4) kstep(A0, B1, A1, B2, cl(kt + 6), cl(kt + 7));
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // the refetches have landed before the epilogue reuses LDS
  // the MFMAs are assembly to the compiler, which therefore does not count their latency: let the last
  // one retire before anything reads an accumulator
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_nop 7\n\ts_nop 7");
  __builtin_amdgcn_sched_barrier(0);

  finish(acc, wave == 0 ? A0 : wave == 1 ? A1 : wave == 2 ? B0 : B1, wave, lane);
}

struct NoHook {
  __device__ __forceinline__ void operator()(int, uint32_t, uint32_t, const u32x4&) const {}
};

// The tile written as BF16 (one RNE) to y[(m0 + r) * ldy + n0 + c]; hook(it, row, col, v) is called for every
// 16-byte group on its way out: a wavefront writes its 128 x 128 part in 32 steps `it` of 4 rows,
// lane = (row % 4, col / 8).
template <bool A_OC, bool B_OC, class Hook>
__device__ __forceinline__ void gemm256_core(const uint16_t* __restrict__ a, uint32_t lda,
                                             const uint16_t* __restrict__ b, uint32_t ldb, uint16_t* __restrict__ y,
                                             uint32_t ldy, uint32_t nk, uint32_t m0, uint32_t n0, Hook&& hook) {
  gemm256_accumulate<A_OC, B_OC>(a, lda, b, ldb, nk, m0, n0, [&](f32x4 (&acc)[8][8], uint16_t* cs, uint32_t wave, uint32_t lane) {
    uint16_t* yw = y + (size_t)(m0 + 128 * (wave >> 1)) * ldy + n0 + 128 * (wave & 1);
    epilogue_bf16_half(*reinterpret_cast<const f32x4 (*)[4][8]>(&acc[0]), 0, cs, yw, ldy, lane, hook);
    epilogue_bf16_half(*reinterpret_cast<const f32x4 (*)[4][8]>(&acc[4]), 1, cs, yw, ldy, lane, hook);
  });
}

}  // namespace gws
