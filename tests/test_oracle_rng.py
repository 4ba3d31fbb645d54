"""Pins of the oracle's random-bit source and bit->R map (paper Sec. 3.4, Eq. 9, Eq. 10).

None of these tests touches a GPU or the product library.
"""
import os
from fractions import Fraction

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_rows(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_philox_known_answer_vectors():
    # Published vectors of the SC'11 generator; a wrong constant, a swapped
    # multiplier or a mis-ordered output word fails all three.
    for row in _read_rows("philox4x32_10_kat.txt"):
        v = [int(x, 16) for x in row]
        assert oracle.philox4x32(v[0:4], v[4:6]) == v[6:10]


def test_philox_rounds_and_counter_sensitivity():
    base = oracle.philox4x32([1, 2, 3, 4], [5, 6])
    assert oracle.philox4x32([1, 2, 3, 4], [5, 6], rounds=9) != base
    for pos in range(4):
        c = [1, 2, 3, 4]
        c[pos] ^= 1
        other = oracle.philox4x32(c, [5, 6])
        # avalanche: about half of the 128 output bits flip
        flips = sum(bin(a ^ b).count("1") for a, b in zip(base, other))
        assert 32 <= flips <= 96


def _eq10_exact():
    """Eq. 10 evaluated exactly, from the printed expressions."""
    p2 = Fraction(3, 4) * Fraction(1, 2 ** 9)               # each sign
    p1 = Fraction(3, 4) ** 2 * Fraction(1, 4) * (1 - 2 * p2)  # each sign; Pr(+-2) = both signs
    p0 = 1 - 2 * p1 - 2 * p2
    return p2, p1, p0


def test_eq10_reading_matches_printed_approximations():
    # The only reading of Eq. 10 that reproduces all three printed figures.
    vals = {k: float(v) for k, v in _read_rows("eq10_distribution.txt")}
    p2, p1, p0 = _eq10_exact()
    assert abs(1 / float(p2) - vals["inv_p2"]) < 0.05
    assert abs(1 / float(p1) - vals["inv_p1"]) < 0.05
    assert abs(float(p0) - vals["p0"]) < 0.0005
    # the other reading of "(1 - Pr(+-2))" (one sign only) misses 0.717 -> 0.7162
    p1_alt = Fraction(3, 4) ** 2 * Fraction(1, 4) * (1 - p2)
    assert abs(float(1 - 2 * p1_alt - 2 * p2) - vals["p0"]) > abs(float(p0) - vals["p0"])


def test_bits_to_r_exhaustive_matches_eq10():
    # 16 bits per element is the least that realises Eq. 10 exactly, so all 65 536
    # inputs can be enumerated: the counts ARE the distribution.
    counts = {}
    for b in range(1 << 16):
        code = oracle.nibbles_to_code(b & 15, (b >> 4) & 15, (b >> 8) & 15, (b >> 12) & 15)
        assert code in (0, 1, 2, 8, 9, 10)          # sign-magnitude, magnitude 3 never occurs
        r = oracle.code_to_r(code)
        counts[r] = counts.get(r, 0) + 1
    p2, p1, p0 = _eq10_exact()
    assert counts[2] == counts[-2] == p2 * 65536 == 96
    assert counts[1] == counts[-1] == p1 * 65536 == 9189
    assert counts[0] == p0 * 65536 == 46966


def test_code_to_r_is_sign_magnitude():
    assert [oracle.code_to_r(c) for c in (0, 1, 2, 8, 9, 10)] == [0, 1, 2, 0, -1, -2]


def test_noise_packed_and_unpacked_agree():
    r, packed = oracle.noise(37, 45, seed=123, step=7)
    assert packed.shape == (37, 6)
    for i in range(37):
        for j in range(45):
            code = (int(packed[i, j >> 3]) >> (4 * (j & 7))) & 0xF
            assert oracle.code_to_r(code) == r[i, j]


def test_noise_uses_counter_col_group_row_step_and_seed_key():
    # The words behind element (i, j) are Philox(ctr=(j>>3, i, step_lo, step_hi), key=seed).
    seed, step = 0x0123456789ABCDEF, 0x00000002_00000005
    r, packed = oracle.noise(3, 24, seed, step)
    for i in range(3):
        for cg in range(3):
            x = oracle.philox4x32([cg, i, step & 0xFFFFFFFF, step >> 32], [seed & 0xFFFFFFFF, seed >> 32])
            word = 0
            for k in range(8):
                # even elements read the low 16-bit half of each word, odd ones the high half
                sh = 4 * (k // 2) + 16 * (k % 2)
                n = [(xx >> sh) & 0xF for xx in x]
                word |= oracle.nibbles_to_code(*n) << (4 * k)
            assert word == int(packed[i, cg])
    assert sorted(oracle.element_nibble(k) for k in range(8)) == list(range(8))


def test_noise_moments_large_sample():
    # >= 6.7e7 samples against the closed-form moments of Eq. 10, each within 5 sigma.
    n_side = 8192
    r, _ = oracle.noise(n_side, n_side, seed=oracle.derive_seed(0, 0), step=0)
    n = r.size
    p2, p1, p0 = map(float, _eq10_exact())
    var = 2 * p1 + 8 * p2
    m4 = 2 * p1 + 32 * p2
    assert abs(var - 19146 / 65536) < 1e-12
    r64 = r.astype(np.int64)
    mean = r64.mean()
    assert abs(mean) < 5 * np.sqrt(var / n)
    r2 = (r64 ** 2).mean()
    assert abs(r2 - var) < 5 * np.sqrt((m4 - var ** 2) / n)
    e_abs = np.abs(r64).mean()
    assert abs(e_abs - (2 * p1 + 4 * p2)) < 5 * np.sqrt((var - (2 * p1 + 4 * p2) ** 2) / n)
    # chi-square over the 5 cells (4 dof): 99.999 % quantile is 28.5
    obs = np.array([(r == v).sum() for v in (-2, -1, 0, 1, 2)], dtype=np.float64)
    exp = np.array([p2, p1, p0, p1, p2]) * n
    chi2 = ((obs - exp) ** 2 / exp).sum()
    assert chi2 < 28.5
    assert abs(obs[2] / n - 0.7166443) < 5 * np.sqrt(p0 * (1 - p0) / n)
    assert set(np.unique(r).tolist()) == {-2, -1, 0, 1, 2}


def test_noise_independence_spot_checks():
    # neighbours in a row (same Philox call, adjacent nibbles), in a column, across
    # adjacent steps and adjacent seeds: correlation of R and of |R| within 5 sigma.
    n_side = 2048
    a, _ = oracle.noise(n_side, n_side, seed=11, step=3)
    b, _ = oracle.noise(n_side, n_side, seed=11, step=4)
    c, _ = oracle.noise(n_side, n_side, seed=12, step=3)
    af = a.astype(np.float64)

    def corr(x, y):
        x = x - x.mean()
        y = y - y.mean()
        return float((x * y).mean() / np.sqrt((x * x).mean() * (y * y).mean()))

    pairs = [(af[:, :-1], af[:, 1:]), (af[:-1, :], af[1:, :]),
             (af, b.astype(np.float64)), (af, c.astype(np.float64)),
             (af[:, :-8], af[:, 8:])]
    for x, y in pairs:
        bound = 5 / np.sqrt(x.size)
        assert abs(corr(x, y)) < bound
        assert abs(corr(np.abs(x), np.abs(y))) < bound
    assert (a != b).mean() > 0.3 and (a != c).mean() > 0.3


def test_noise_is_a_pure_function_of_seed_and_step():
    a, pa = oracle.noise(64, 64, seed=5, step=9)
    _ = oracle.noise(64, 64, seed=6, step=1)
    b, pb = oracle.noise(64, 64, seed=5, step=9)
    assert (a == b).all() and (pa == pb).all()
    # a sub-tensor sees the same noise as the full tensor at the same coordinates
    c, _ = oracle.noise(32, 40, seed=5, step=9)
    assert (c == a[:32, :40]).all()


def test_derive_seed():
    s = {oracle.derive_seed(0, i) for i in range(1000)}
    assert len(s) == 1000
    assert oracle.derive_seed(0, 1) != oracle.derive_seed(1, 0)
    # definition: low 64 bits of Philox(ctr=(id_lo, id_hi, 'GWS1', 0), key=user seed)
    u, t = 0xDEADBEEF12345678, 0x1_00000002
    x = oracle.philox4x32([t & 0xFFFFFFFF, t >> 32, 0x47575331, 0], [u & 0xFFFFFFFF, u >> 32])
    assert oracle.derive_seed(u, t) == x[0] | (x[1] << 32)
