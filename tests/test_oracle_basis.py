"""Pins of the oracle's comparison noise bases (paper Sec. 4: the "DiffQ" extension with a BF16 U(-0.5, 0.5) basis;
Sec. 4 "Overhead": the "bm" baseline, round(N(0,1)/2) from a Box-Muller transform).

What fixes them independently of the oracle's own code:
  uniform     the 256 values enumerated: exact mean 0, exact variance (1 - 2^-16)/12, all BF16 members of (-0.5, 0.5),
              equally spaced; the byte an element owns recomposed in Python from Philox outputs (pinned by the SC'11
              vectors); bf16(R * s) against torch's CPU bfloat16 product
  Box-Muller  both normals against the fp64 textbook formula on random and extreme words; z0^2 + z1^2 = -2 ln u1;
              the cell probabilities of round(z / 2) against erf on 2^24 samples (chi-square); the word / half / element
              assignment recomposed in Python
  forward     Eq. 3 recomposed from torch CPU bfloat16 arithmetic for integer b_t (power-of-two scale)
  backward    Eq. 4's definition evaluated with numpy in fp64
CPU only."""
import math

import numpy as np
import pytest
import torch

import oracle
from test_oracle_sample import bf16_val, block_absmax, expand, to_bits

U, BM = oracle.BASIS_UNIFORM, oracle.BASIS_BOX_MULLER
LN2 = math.log(2.0)


# ---------------------------------------------------------------- uniform
def test_uniform_values_enumerated():
    vals = bf16_val(np.array([oracle.uniform_bf16(b) for b in range(256)], dtype=np.uint16))
    assert (np.diff(vals) == 1.0 / 256).all()                       # equally spaced, ascending in the byte
    assert vals[0] == -255.0 / 512 and vals[-1] == 255.0 / 512      # inside (-0.5, 0.5)
    assert vals.sum() == 0.0 and (vals == -vals[::-1]).all()        # mean exactly 0, symmetric
    assert np.mean(vals ** 2) == (1.0 - 2.0 ** -16) / 12.0          # variance of U(-0.5, 0.5) up to the grid term
    # BF16 members: converting through torch's bfloat16 changes nothing
    assert (to_bits(vals) == np.array([oracle.uniform_bf16(b) for b in range(256)], dtype=np.uint16)).all()


def test_uniform_element_owns_byte_k_mod_4_of_word_k_div_4():
    seed, step = oracle.derive_seed(3, 1), 5
    r = oracle.noise_basis(6, 48, seed, step, U, row0=32, col0=64)
    for i in range(6):
        for j in range(48):
            x = oracle.philox4x32([(64 + j) >> 3, 32 + i, step & 0xFFFFFFFF, step >> 32], [seed & 0xFFFFFFFF, seed >> 32])
            k = j & 7
            byte = (x[k >> 2] >> (8 * (k & 3))) & 0xFF
            assert r[i, j] == (2 * byte - 255) / 512.0


def test_bf16_mul_matches_torch():
    rng = np.random.default_rng(1)
    a = rng.integers(0, 65536, 200000).astype(np.uint16)
    b = rng.integers(0, 65536, 200000).astype(np.uint16)
    fin = (((a >> 7) & 0xFF) != 0xFF) & (((b >> 7) & 0xFF) != 0xFF)
    # keep the products inside fp32's normal range, where the two-step rounding argument holds
    ea, eb = ((a >> 7) & 0xFF).astype(int), ((b >> 7) & 0xFF).astype(int)
    ok = fin & (ea + eb > 127 - 100) & (ea + eb < 127 + 350 - 127)
    a, b = a[ok], b[ok]
    ta = torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
    tb = torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16)
    want = (ta * tb).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.bf16_mul(int(x), int(y)) for x, y in zip(a[:20000], b[:20000])], dtype=np.uint16)
    fin2 = ((want[:20000] >> 7) & 0xFF) != 0xFF
    assert (got[fin2] == want[:20000][fin2]).all()
    assert oracle.bf16_mul(0x3F80, 0x3F81) == 0x3F81                        # 1 * x = x
    assert oracle.bf16_mul(0x3FC0, 0x3FC0) == 0x4010                        # 1.5^2 = 2.25 exactly
    assert oracle.bf16_mul(0x3F81, 0x3F81) == 0x3F82                        # (1 + 2^-7)^2 = 1 + 2^-6 + 2^-14 -> 1.015625
    assert oracle.bf16_mul(0x3EFF, 0x3F81) == 0x3F00                        # 0.498046875 * 1.0078125 = 0.50194: nearest is 0.5
    v = bf16_val(np.array([0x3EFF, 0x3F81], dtype=np.uint16))
    exact = v[0] * v[1]
    cands = bf16_val(np.array([0x3EFF, 0x3F00, 0x3F01], dtype=np.uint16))
    assert bf16_val(np.array([oracle.bf16_mul(0x3EFF, 0x3F81)], dtype=np.uint16))[0] == cands[np.argmin(np.abs(cands - exact))]


# ---------------------------------------------------------------- Box-Muller
def reference_normals(words):
    w = np.asarray(words, dtype=np.uint64)
    u1 = ((w & 0xFFFF).astype(np.float64) + 0.5) / 65536.0
    u2 = ((w >> 16).astype(np.float64) + 0.5) / 65536.0
    r = np.sqrt(-2.0 * np.log(u1))
    return r * np.cos(2.0 * np.pi * u2), r * np.sin(2.0 * np.pi * u2), u1


def test_box_muller_matches_the_fp64_formula():
    rng = np.random.default_rng(2)
    words = np.concatenate([rng.integers(0, 2 ** 32, 1 << 20, dtype=np.uint64).astype(np.uint32),
                            np.array([0, 0xFFFFFFFF, 0x0000FFFF, 0xFFFF0000, 0x3FFF0000, 0x40000000, 0x7FFF8000,
                                      0x80000001, 0xBFFF0000, 0xC0000000], dtype=np.uint32)])
    # every value of u1 and every quadrant boundary of u2 at least once
    words = np.concatenate([words, np.arange(65536, dtype=np.uint32) | (rng.integers(0, 65536, 65536).astype(np.uint32) << 16),
                            (np.arange(65536, dtype=np.uint32) << 16) | rng.integers(0, 65536, 65536).astype(np.uint32)])
    z = oracle.box_muller(words).astype(np.float64)
    z0, z1, u1 = reference_normals(words)
    assert np.abs(z[:, 0] - z0).max() < 2e-6 and np.abs(z[:, 1] - z1).max() < 2e-6
    assert np.abs(z[:, 0] ** 2 + z[:, 1] ** 2 + 2.0 * np.log(u1)).max() < 2e-5       # the pair lies on the circle of radius r
    assert np.abs(z).max() < 4.86                                                     # 16-bit u1: round(z/2) stays within +-2


def test_box_muller_cells_match_the_rounded_normal():
    # cell probabilities of round(N(0,1)/2): boundaries |z| = 1, 3 (ties to even make no difference in probability)
    rows, cols = 4096, 4096
    r = oracle.noise_basis(rows, cols, oracle.derive_seed(7, 0), 1, BM).astype(np.int64)
    n = rows * cols
    Phi = lambda x: 0.5 * (1.0 + math.erf(x / math.sqrt(2.0)))
    p0, p1, p2 = 2 * Phi(1) - 1, Phi(3) - Phi(1), 1 - Phi(3)
    expect = np.array([p2, p1, p0, p1, p2]) * n
    count = np.array([(r == v).sum() for v in (-2, -1, 0, 1, 2)])
    assert count.sum() == n                                                          # nothing outside {-2, ..., 2}
    chi2 = ((count - expect) ** 2 / expect).sum()
    assert chi2 < 30.0, (count, expect)                                              # 4 d.o.f.; P(chi2 > 30) ~ 5e-6
    # moments of the rounded normal: mean 0, variance sum k^2 p_k
    assert abs(r.mean()) < 5 * math.sqrt((2 * p1 + 8 * p2) / n)
    assert abs((r ** 2).mean() - (2 * p1 + 8 * p2)) < 1e-3
    # neighbours in a pair (cos and sin branch of one transform) are uncorrelated
    assert abs(np.mean(r[:, 0::2] * r[:, 1::2])) < 1e-3


def test_box_muller_pair_d_takes_word_d_cos_then_sin():
    seed, step = oracle.derive_seed(3, 2), 9
    r = oracle.noise_basis(4, 40, seed, step, BM, row0=64, col0=32)
    for i in range(4):
        for j in range(40):
            x = oracle.philox4x32([(32 + j) >> 3, 64 + i, step, 0], [seed & 0xFFFFFFFF, seed >> 32])
            k = j & 7
            z0, z1, _ = reference_normals([x[k >> 1]])
            z = (z0 if (k & 1) == 0 else z1)[0]
            if abs(abs(z) - 1.0) > 1e-4 and abs(abs(z) - 3.0) > 1e-4:                 # away from a cell boundary
                assert r[i, j] == np.round(z / 2.0), (i, j, z)


# ---------------------------------------------------------------- forward / backward with a basis
def library_forward_basis(w_bits, bt_int, basis, seed, step):
    rows, cols = w_bits.shape
    a = block_absmax(bf16_val(w_bits), rows, cols)
    s32 = (a * np.exp2(1.0 - bt_int)).astype(np.float32)
    s16 = torch.from_numpy(expand(s32, rows, cols)).to(torch.bfloat16)
    r = torch.from_numpy(oracle.noise_basis(rows, cols, seed, step, basis)).to(torch.bfloat16)    # exact: BF16 members
    w_t = torch.from_numpy(w_bits.view(np.int16).copy()).view(torch.bfloat16)
    w_hat = w_t + r * s16                                                            # BF16 product, then BF16 sum
    return w_hat.view(torch.int16).numpy().view(np.uint16), s32


@pytest.mark.parametrize("basis", [U, BM])
@pytest.mark.parametrize("shape", [(96, 160), (70, 45)])
def test_forward_with_a_basis_vs_library_composition(basis, shape):
    rows, cols = shape
    rng = np.random.default_rng(rows)
    w = to_bits(rng.standard_normal((rows, cols)) * 0.02)
    nbr, nbc = oracle.n_blocks(rows, cols)
    bt = rng.integers(3, 9, size=(nbr, nbc)).astype(np.float32)
    seed = oracle.derive_seed(1, rows)
    q, scale = oracle.sample_fwd(w, bt, oracle.FMT_BF16, seed, 2, basis=basis)
    want, s32 = library_forward_basis(w, bt, basis, seed, 2)
    assert (scale == s32).all()
    assert (q == want).all()
    # and the basis matters: the bit basis gives another result
    q0, _ = oracle.sample_fwd(w, bt, oracle.FMT_BF16, seed, 2)
    assert (q0 != q).any()


@pytest.mark.parametrize("basis", [U, BM])
def test_forward_cast_applies_after_the_add(basis):
    rng = np.random.default_rng(5)
    w = to_bits(rng.standard_normal((64, 64)) * 0.02)
    bt = np.full((2, 2), 4.0, np.float32)
    q16, _ = oracle.sample_fwd(w, bt, oracle.FMT_BF16, 9, 0, basis=basis)
    q8, _ = oracle.sample_fwd(w, bt, oracle.FMT_FP8_E4M3, 9, 0, basis=basis)
    a = block_absmax(bf16_val(w), 64, 64)
    for bi in range(2):
        for bj in range(2):
            Ea = int(np.floor(np.log2(a[bi, bj])))
            blk = (slice(bi * 32, bi * 32 + 32), slice(bj * 32, bj * 32 + 32))
            assert (oracle.cast_n(q16[blk].ravel(), Ea, oracle.FMT_FP8_E4M3) == q8[blk].ravel()).all()


@pytest.mark.parametrize("basis", [U, BM])
def test_backward_with_a_basis_matches_the_definition(basis):
    rows, cols = 70, 100
    rng = np.random.default_rng(6)
    g = to_bits(rng.standard_normal((rows, cols)) * 1e-3)
    nbr, nbc = oracle.n_blocks(rows, cols)
    scale = (rng.random((nbr, nbc)) * 1e-3 + 1e-5).astype(np.float32)
    seed = oracle.derive_seed(2, 2)
    dw, dbt, asum = oracle.sample_bwd(g, scale, seed, 3, basis=basis)
    assert (dw == g).all()
    gr = bf16_val(g) * oracle.noise_basis(rows, cols, seed, 3, basis).astype(np.float64)
    for bi in range(nbr):
        for bj in range(nbc):
            blk = gr[bi * 32:bi * 32 + 32, bj * 32:bj * 32 + 32]
            assert np.isclose(dbt[bi, bj], -LN2 * float(scale[bi, bj]) * blk.sum(), rtol=1e-12, atol=1e-300)
            assert np.isclose(asum[bi, bj], LN2 * float(scale[bi, bj]) * np.abs(blk).sum(), rtol=1e-12)


def test_basis_zero_is_the_bit_basis():
    rng = np.random.default_rng(8)
    w = to_bits(rng.standard_normal((40, 72)) * 0.02)
    bt = (4.0 + 5.0 * rng.random((2, 3))).astype(np.float32)
    a = oracle.sample_fwd(w, bt, oracle.FMT_FP6_E3M2, 5, 1)
    b = oracle.sample_fwd(w, bt, oracle.FMT_FP6_E3M2, 5, 1, basis=oracle.BASIS_BITS)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()
    r, _ = oracle.noise(40, 72, 5, 1)
    assert (oracle.noise_basis(40, 72, 5, 1, oracle.BASIS_BITS) == r).all()
