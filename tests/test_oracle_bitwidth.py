"""Pins of the oracle's bitwidth parametrisation (paper Sec. 3.6 "Bitwidth", Eq. 11 and Eq. 12).

The loss of Eq. 12 and the map of Eq. 11 are written out here in fp64 from their definitions
and differentiated numerically; the oracle's gradient has to agree.  CPU only."""
import numpy as np

import oracle
from paper_2505_11170_amd import synth
from test_oracle_sample import bf16_val, block_absmax, expand


def test_eq11_end_points_and_midpoint():
    # b_i = 1 gives b_init (the paper initialises b_i with 1), b_i = 0 gives b_target
    for b_init, b_target in [(6.0, 4.0), (8.0, 4.0), (5.0, 5.0), (4.0, 9.0)]:
        bi = np.array([1.0, 0.0, 0.5, -0.5, 2.0], dtype=np.float32)
        bt = oracle.bitwidth(bi, b_init, b_target)
        d = b_init - b_target
        assert bt.dtype == np.float32
        assert bt.tolist() == [b_init, b_target, b_target + 0.5 * d, b_target - 0.5 * d, b_target + 2 * d]


def test_eq11_is_fp32_rounding_of_the_real_formula():
    rng = np.random.default_rng(3)
    bi = rng.uniform(-0.5, 1.5, 20000).astype(np.float32)
    b_init, b_target = np.float32(6.3), np.float32(3.9)
    bt = oracle.bitwidth(bi, float(b_init), float(b_target))
    exact = float(b_target) + bi.astype(np.float64) * (float(b_init) - float(b_target))
    # three fp32 roundings (difference, product, sum) of magnitudes below 16: within 3 * 2^-21
    assert np.abs(bt.astype(np.float64) - exact).max() <= 3 * 2.0 ** -21
    # and it is exactly the sequence difference -> product -> sum in fp32
    delta = np.float32(b_init - b_target)
    assert np.array_equal(bt, (b_target + (bi * delta).astype(np.float32)).astype(np.float32))


def _loss_eq12(bi, c, b_init, b_target, lam, m):
    """L' of Eq. 12 for one layer whose task loss is linear in b_t: L = sum(c * b_t)."""
    bt = b_target + bi * (b_init - b_target)
    return (c * bt).sum() + lam * np.abs(bt - b_target).sum() / m


def test_eq12_gradient_matches_finite_differences():
    rng = np.random.default_rng(5)
    n, m = 40, 100                      # 40 blocks handed in, of a layer of 100 blocks
    b_init, b_target, lam = 6.0, 4.0, 0.37
    bi = rng.uniform(0.1, 1.2, n)
    bi[::3] *= -1.0                     # both sides of b_target
    c = rng.normal(size=n)              # dL/db_t
    grad = oracle.bitwidth_grad(bi.astype(np.float32), c, b_init, b_target, lam, m)
    bi32 = bi.astype(np.float32).astype(np.float64)
    h = 1e-5
    for k in range(n):
        e = np.zeros(n)
        e[k] = h
        fd = (_loss_eq12(bi32 + e, c, b_init, b_target, lam, m) -
              _loss_eq12(bi32 - e, c, b_init, b_target, lam, m)) / (2 * h)
        assert abs(grad[k] - fd) <= 1e-8 * max(1.0, abs(fd)), (k, grad[k], fd)


def test_eq12_special_cases():
    c = np.array([0.25, -1.5, 3.0])
    bi = np.array([1.0, 0.0, -1.0], dtype=np.float32)
    # lambda = 0: the chain rule through Eq. 11 alone
    assert np.array_equal(oracle.bitwidth_grad(bi, c, 6.0, 4.0, 0.0, 7), 2.0 * c)
    # at b_t = b_target the subgradient of |.| is taken as 0; the sign follows b_t - b_target
    g = oracle.bitwidth_grad(bi, c, 6.0, 4.0, 0.7, 7)
    assert np.allclose(g, 2.0 * (c + 0.7 / 7 * np.array([1.0, 0.0, -1.0])), rtol=1e-15, atol=0)
    # b_init below b_target flips b_delta, and with it the side b_i = 1 lies on
    g = oracle.bitwidth_grad(bi, c, 4.0, 6.0, 0.7, 7)
    assert np.allclose(g, -2.0 * (c + 0.7 / 7 * np.array([-1.0, 0.0, 1.0])), rtol=1e-15, atol=0)
    # b_init == b_target: b_t does not depend on b_i
    assert np.array_equal(oracle.bitwidth_grad(bi, c, 5.0, 5.0, 0.7, 7), np.zeros(3))


def test_full_chain_finite_difference_through_eq3():
    # L'(b_i) = sum(g .* w_hat(b_t(b_i))) + lambda * sum|b_t - b_target| / m on the real-valued Eq. 3, R fixed
    rows, cols = 64, 96
    t = synth.make_tensor(11, rows, cols)
    w, g = synth.bits(t["w"]), synth.bits(t["g"])
    rng = np.random.default_rng(11)
    bi = rng.uniform(0.2, 1.1, (2, 3)).astype(np.float32)
    b_init, b_target, lam, m = 7.0, 4.0, 1e-6, 6
    seed = 99
    r, _ = oracle.noise(rows, cols, seed, 0)
    wv, gv = bf16_val(w), bf16_val(g)
    a = block_absmax(wv, rows, cols)

    def loss_blocks(b_i):
        b = b_target + b_i * (b_init - b_target)
        w_hat = wv + r * expand(a * np.exp2(1.0 - b), rows, cols)
        return (gv * w_hat).reshape(2, 32, 3, 32).sum(axis=(1, 3)) + lam * np.abs(b - b_target) / m
    h = 1e-4
    bi64 = bi.astype(np.float64)
    fd = (loss_blocks(bi64 + h) - loss_blocks(bi64 - h)) / (2 * h)
    bt = oracle.bitwidth(bi, b_init, b_target)
    _, scale = oracle.sample_fwd(w, bt, 0, seed, 0)
    _, dbt, asum = oracle.sample_bwd(g, scale, seed, 0)
    dbi = oracle.bitwidth_grad(bi, dbt, b_init, b_target, lam, m)
    assert np.allclose(dbi, fd, rtol=5e-6, atol=3e-7 * asum.max())
    # the loss term is visible: without it the gradients differ by (b_init - b_target) * lambda / m
    dbi0 = oracle.bitwidth_grad(bi, dbt, b_init, b_target, 0.0, m)
    assert np.allclose(dbi - dbi0, (b_init - b_target) * lam / m, rtol=1e-9, atol=0)
