"""Pins of the oracle's arithmetic: 2^(1-b_t), the BF16 add, the fp_{e,m} casts
(paper Sec. 3.2 Eq. 3, Sec. 3.3).  CPU only; checked against library routines
(torch CPU bfloat16 / float8_e4m3fn, numpy fp64) and brute force."""
import numpy as np
import torch

import oracle

ALL16 = np.arange(1 << 16, dtype=np.uint16)


def bf16_val(bits):
    """uint16 patterns -> float64 values (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def finite_mask(bits):
    return (np.asarray(bits) & 0x7F80) != 0x7F80


# ---------------------------------------------------------------- exp2
def test_exp2_exact_on_integers():
    for n in range(-40, 41):
        assert oracle.exp2(float(n)) == 2.0 ** n


def test_exp2_within_one_ulp_of_fp64():
    rng = np.random.default_rng(0)
    t = np.concatenate([rng.uniform(-14, 3, 2_000_000), np.linspace(-9, -2, 500_001)]).astype(np.float32)
    got = oracle.exp2_n(t).astype(np.float64)
    true = np.exp2(t.astype(np.float64))
    ulp = np.spacing(true.astype(np.float32)).astype(np.float64)
    assert np.abs(got - true).max() <= 1.0 * ulp.max() and (np.abs(got - true) / ulp).max() < 1.0


def test_exp2_monotone_on_the_used_range():
    t = np.sort(np.random.default_rng(1).uniform(-9, -2, 1_000_000).astype(np.float32))
    p = oracle.exp2_n(t)
    assert (np.diff(p) >= 0).all()


# ---------------------------------------------------------------- BF16 rounding / add
def test_bf16_rne_matches_torch():
    rng = np.random.default_rng(2)
    u = rng.integers(0, 1 << 32, 300_000, dtype=np.uint64).astype(np.uint32)
    u = u[(u & 0x7F800000) != 0x7F800000]
    f = u.view(np.float32)
    want = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.bf16_rne(float(x)) for x in f[:50_000]], dtype=np.uint16)
    assert (got == want[:50_000]).all()
    # ties: 1 + 2^-8 -> 1 (even), 1.0078125 + 2^-8 -> 1.015625
    assert oracle.bf16_rne(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle.bf16_rne(1.0078125 + 2.0 ** -8) == 0x3F82


def _torch_bf16_add(a_bits, b_bits):
    a = torch.from_numpy(a_bits.view(np.int16).copy()).view(torch.bfloat16)
    b = torch.from_numpy(b_bits.view(np.int16).copy()).view(torch.bfloat16)
    return (a + b).view(torch.int16).numpy().view(np.uint16)


def _check_add(a_bits, b_bits):
    got = oracle.bf16_add_n(a_bits, b_bits)
    want = _torch_bf16_add(a_bits, b_bits)
    # independent route 2: exact sum in fp64 (bf16 + bf16 is exact in fp64 unless the
    # exponents differ by > 44, where the smaller addend cannot matter), rounded once
    s = bf16_val(a_bits) + bf16_val(b_bits)
    ok = np.isfinite(s) & (np.abs(s) < 3.3e38)
    # compare as values where finite; -0/+0 must match as bits too
    assert (got[ok] == want[ok]).all(), np.flatnonzero(got[ok] != want[ok])[:5]
    gv = bf16_val(got[ok])
    ulp_gap = np.abs(gv - s[ok])
    nxt = np.spacing(np.abs(gv).astype(np.float32)).astype(np.float64) * 2 ** 16  # bf16 ulp
    assert (ulp_gap <= nxt / 2 + 1e-300).all()


def test_bf16_add_random_pairs_vs_torch():
    rng = np.random.default_rng(3)
    a = rng.integers(0, 1 << 16, 3_000_000).astype(np.uint16)
    b = rng.integers(0, 1 << 16, 3_000_000).astype(np.uint16)
    m = finite_mask(a) & finite_mask(b)
    _check_add(a[m], b[m])


def test_bf16_add_close_exponents_vs_torch():
    # random pairs rarely have nearby exponents; force exponent gaps 0..12, both signs,
    # where alignment, cancellation and ties actually happen
    rng = np.random.default_rng(4)
    n = 2_000_000
    ea = rng.integers(1, 250, n)
    gap = rng.integers(0, 13, n)
    eb = np.clip(ea - gap, 0, 254)
    a = ((rng.integers(0, 2, n) << 15) | (ea << 7) | rng.integers(0, 128, n)).astype(np.uint16)
    b = ((rng.integers(0, 2, n) << 15) | (eb << 7) | rng.integers(0, 128, n)).astype(np.uint16)
    _check_add(a, b)


def test_bf16_add_exhaustive_against_fixed_operands():
    # every BF16 pattern added to a handful of fixed operands, subnormals and zeros included
    for fixed in (0x0000, 0x8000, 0x3F80, 0xBF80, 0x3E00, 0x3C00, 0x0001, 0x8001, 0x007F, 0x0080,
                  0x3B80, 0xBB80, 0x7F00, 0x3F81, 0x3EFF):
        a = ALL16[finite_mask(ALL16)]
        b = np.full_like(a, fixed)
        _check_add(a, b)
        _check_add(b, a)


def test_bf16_add_hand_ties():
    one, eps = 0x3F80, 0x3B80            # 1.0, 2^-8 (half an ulp of 1.0)
    assert oracle.bf16_add(one, eps) == 0x3F80           # tie -> even
    assert oracle.bf16_add(0x3F81, eps) == 0x3F82        # 1.0078125 + 2^-8 -> 1.015625
    assert oracle.bf16_add(one, 0xBF80) == 0x0000        # x - x = +0
    assert oracle.bf16_add(0x8000, 0x8000) == 0x8000     # -0 + -0 = -0
    assert oracle.bf16_add(0x8000, 0x0000) == 0x0000     # -0 + +0 = +0
    assert oracle.bf16_add(0x3F80, 0x8000) == 0x3F80     # x + -0 = x


# ---------------------------------------------------------------- casts
FORMATS = {
    oracle.FMT_FP8_E4M3: dict(emax=8, emin=-6, m=3, maxv=448.0),   # OCP FP8 E4M3: no Inf, max 1.75*2^8
    oracle.FMT_FP6_E3M2: dict(emax=4, emin=-2, m=2, maxv=28.0),    # OCP MX FP6 E3M2: no Inf/NaN, max 1.75*2^4
}


def code_set(fmt):
    """All non-negative finite values of the format, enumerated from its bit layout."""
    p = FORMATS[fmt]
    ebits = 4 if fmt == oracle.FMT_FP8_E4M3 else 3
    bias = 7 if fmt == oracle.FMT_FP8_E4M3 else 3
    vals = []
    for e in range(1 << ebits):
        for man in range(1 << p["m"]):
            if fmt == oracle.FMT_FP8_E4M3 and e == 15 and man == 7:
                continue  # NaN
            if e == 0:
                v = man * 2.0 ** (1 - bias - p["m"])
            else:
                v = (1 + man / (1 << p["m"])) * 2.0 ** (e - bias)
            vals.append(v)
    vals = np.array(vals)
    assert vals.max() == p["maxv"] and (np.diff(vals) > 0).all()
    assert vals[1] == 2.0 ** (p["emin"] - p["m"])
    return vals


def brute_force_cast(v, Ea, fmt):
    """Nearest member of X * code_set with ties to the even code, saturating."""
    p = FORMATS[fmt]
    X = 2.0 ** (Ea + 1 - p["emax"])
    grid = code_set(fmt) * X
    av = np.abs(v)
    idx = np.searchsorted(grid, av)          # grid[idx-1] < av <= grid[idx]
    idx = np.clip(idx, 1, len(grid) - 1)
    lo, hi = grid[idx - 1], grid[idx]
    d_lo, d_hi = av - lo, hi - av
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & ((idx % 2) == 0))   # code index parity = mantissa lsb
    out = np.where(pick_hi, hi, lo)
    out = np.where(av >= grid[-1], grid[-1], out)
    return np.copysign(out, v)


def test_cast_bf16_is_identity():
    assert (oracle.cast_n(ALL16, 0, oracle.FMT_BF16) == ALL16).all()


def test_cast_exhaustive_vs_brute_force():
    bits = ALL16[finite_mask(ALL16)]
    v = bf16_val(bits)
    for fmt in FORMATS:
        for Ea in (-20, -7, -6, -1, 0, 1, 5):
            got = oracle.cast_n(bits, Ea, fmt)
            want = brute_force_cast(v, Ea, fmt)
            gv = bf16_val(got)
            assert (gv == want).all(), (fmt, Ea, np.flatnonzero(gv != want)[:5])
            assert ((got & 0x8000) == (bits & 0x8000)).all()       # sign kept, also for zeros


def test_cast_e4m3_vs_torch_float8():
    bits = ALL16[finite_mask(ALL16)]
    v32 = (bits.astype(np.uint32) << 16).view(np.float32)
    for Ea in (-9, -6, 0, 3):
        xe = Ea + 1 - 8
        y = torch.from_numpy(v32.copy()) * (2.0 ** -xe)                  # exact power-of-two scaling
        inr = (y.abs() <= 448.0) & (y.abs() >= 2.0 ** -20)
        q = y.to(torch.float8_e4m3fn).to(torch.float32) * (2.0 ** xe)
        got = bf16_val(oracle.cast_n(bits, Ea, oracle.FMT_FP8_E4M3))
        m = inr.numpy()
        assert (got[m] == q.numpy().astype(np.float64)[m]).all()


def test_cast_outputs_are_representable_and_idempotent():
    bits = ALL16[finite_mask(ALL16)]
    for fmt, p in FORMATS.items():
        for Ea in (-6, 0, 2):
            X = 2.0 ** (Ea + 1 - p["emax"])
            got = oracle.cast_n(bits, Ea, fmt)
            members = set((code_set(fmt) * X).tolist())
            assert set(np.abs(bf16_val(got)).tolist()) <= members
            assert (oracle.cast_n(got, Ea, fmt) == got).all()
            # monotone non-decreasing in the input value
            order = np.argsort(bf16_val(bits), kind="stable")
            assert (np.diff(bf16_val(got)[order]) >= 0).all()


def test_cast_hand_cases():
    # block with max|w| = 1.0: Ea = 0, X_e4m3 = 2^-7, X_e3m2 = 2^-3
    def c(x, fmt):
        b = torch.tensor([x], dtype=torch.float32).to(torch.bfloat16).view(torch.int16).item() & 0xFFFF
        assert bf16_val(np.array([b], dtype=np.uint16))[0] == x          # x must itself be BF16
        return bf16_val(np.array([oracle.cast(b, 0, fmt)], dtype=np.uint16))[0]
    E4, E3 = oracle.FMT_FP8_E4M3, oracle.FMT_FP6_E3M2
    assert c(1.25, E4) == 1.25 and c(1.25, E3) == 1.25
    assert c(0.42578125, E4) == 0.4375 and c(0.42578125, E3) == 0.4375
    assert c(0.30078125, E4) == 0.3125 and c(0.30078125, E3) == 0.3125
    assert c(-0.1171875, E4) == -0.1171875
    assert c(-0.1171875, E3) == -0.125                 # 0.9375*X: tie -> even
    assert c(2.0 ** -8, E4) == 2.0 ** -8
    assert c(2.0 ** -8, E3) == 0.0                     # half of the smallest subnormal: tie -> 0
    assert c(2.0 ** -17, E4) == 0.0
    assert c(3 * 2.0 ** -18, E4) == 2.0 ** -16
    # saturation: E4M3 max is 448 * 2^-7 = 3.5, E3M2 max is 28 * 2^-3 = 3.5
    assert c(4.0, E4) == 3.5 and c(-100.0, E3) == -3.5
