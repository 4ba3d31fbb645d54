"""GPU parity of gws_linear_bwd_w: the weight-gradient GEMM dW = X^T dY with the block reduction of the
paper's Eq. 4 in its epilogue.  dW is checked against the fp64 oracle GEMM (one BF16 rounding + fp32
accumulation in any order); dL/db_t is checked against the oracle's backward pass on the very dW bytes
the GPU produced (the reduction is defined on the rounded BF16 gradient), to the 1e-5 bar."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_11170_amd as gws
from paper_2505_11170_amd import synth
from gpu_util import DEV, assert_dbt_close, ensure_built

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def f64(bits):
    return (np.ascontiguousarray(bits).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def run_case(M, K, N, w_is_nk, idx, step=4, rows_sel=None, pad=0, row0=0, col0=0, split=None):
    """split: None = gws_linear_bwd_w; a number of bytes = gws_linear_bwd_w_ws with a workspace of that size
    (-1: the size gws_linear_bwd_w_workspace_bytes names, which must then be positive)."""
    x = synth.make_activation(idx, M, K)
    dy = (synth.make_activation(idx + 1, M, N).float() * 1e-3).to(torch.bfloat16)   # upstream gradient ~ N(0, 1e-3)
    rows, cols = (N, K) if w_is_nk else (K, N)
    ld = cols + pad
    nbr, nbc = rows // 32, cols // 32
    gen = torch.Generator().manual_seed(9000 + idx)
    scale = (torch.rand(nbr, nbc, generator=gen) * 1e-3 + 1e-5).float()
    seed = oracle.derive_seed(2, idx)
    dw = torch.zeros(rows, ld, dtype=torch.bfloat16, device=DEV)
    dbt = torch.full((nbr, nbc), float("nan"), device=DEV)
    d = gws.TensorDesc(rows=rows, cols=cols, seed=seed, scale=scale.to(DEV), dw=dw, dbt=dbt, ld=ld, row0=row0, col0=col0)
    xg, dyg = x.to(DEV), dy.to(DEV)
    if split is None:
        gws.gws_linear_bwd_w(xg, dyg, d, step, w_is_nk=w_is_nk)
    else:
        want = gws.gws_linear_bwd_w_workspace_bytes(d, M)
        if split < 0:
            assert want > 0, ("no split planned", M, K, N)
            split = want
        ws = torch.full((max(split, 16) // 4,), float("nan"), device=DEV)          # stale contents must not matter
        gws.gws_linear_bwd_w_ws(xg, dyg, d, step, ws[: split // 4], w_is_nk=w_is_nk)
    torch.cuda.synchronize()
    dw_bits = synth.bits(dw)
    assert (dw_bits[:, cols:] == 0).all()                       # padding columns are never written
    # dW against the fp64 GEMM: rows of dW are columns of A (X, or dY for the [N x K] layout)
    a, b = (dy, x) if w_is_nk else (x, dy)
    at = np.ascontiguousarray(synth.bits(a).T)
    sel = None if rows_sel is None else np.asarray(rows_sel)
    y64, yabs, _ = oracle.linear_fwd(at, synth.bits(b), rows_sel=sel)
    got = f64(dw_bits[:, :cols] if sel is None else dw_bits[sel, :cols])
    tol = 2.0 ** -8 * np.abs(y64) + M * 2.0 ** -24 * yabs + 1e-30
    assert (np.abs(got - y64) <= tol).all(), ("dW", M, K, N, w_is_nk)
    # dL/db_t against the oracle's Eq. 4 on the GPU's own dW bytes
    _, ref_dbt, asum = oracle.sample_bwd(np.ascontiguousarray(dw_bits), scale.numpy(), seed, step, cols=cols, row0=row0, col0=col0)
    assert_dbt_close(dbt.cpu().numpy(), ref_dbt, asum, ("dbt", M, K, N, w_is_nk))
    return xg, dyg, d, dw_bits, dbt.cpu().numpy()


@pytest.mark.parametrize("w_is_nk", [False, True])
def test_single_tile_and_several_tiles(w_is_nk):
    run_case(64, 256, 256, w_is_nk, 800)
    run_case(192, 512, 768, w_is_nk, 802, pad=8)
    run_case(128, 768, 256, w_is_nk, 804, row0=256, col0=512)     # a shard: the origin enters the noise counter


def test_every_number_of_k_steps():
    # tokens are the contraction here: 1 .. 13 K-steps of 64 tokens take every path through the prologue, the
    # six-fold unrolled loop and its tail
    for nk in range(1, 14):
        run_case(64 * nk, 256, 256, bool(nk & 1), 840 + 2 * nk)


@pytest.mark.parametrize("w_is_nk", [False, True])
def test_config5_shape(w_is_nk):
    M, K, N = 8192, 2048, 5632
    rows = N if w_is_nk else K
    # one row of dW in every 256-row tile of the weight, at a different 32-row sub-tile each time, plus the ends
    rng = np.random.default_rng(810)
    sel = sorted({0, rows - 1} | {t * 256 + 32 * (t % 8) + int(rng.integers(0, 32)) for t in range(rows // 256)})
    run_case(M, K, N, w_is_nk, 810, rows_sel=sel)


def test_epilogue_agrees_with_the_separate_backward_kernel_and_plain_form():
    xg, dyg, d, dw_bits, dbt = run_case(256, 512, 512, False, 820)
    # the same dW without the reduction
    dw2 = torch.zeros_like(d.dw)
    d2 = gws.TensorDesc(rows=d.rows, cols=d.cols, seed=d.seed, dw=dw2, ld=d.ld)
    gws.gws_linear_bwd_w(xg, dyg, d2, 4)
    # and the separate kernel on those bytes
    dbt3 = torch.zeros_like(d.dbt)
    d3 = gws.TensorDesc(rows=d.rows, cols=d.cols, seed=d.seed, g=d.dw, dw=d.dw, dbt=dbt3, scale=d.scale, ld=d.ld)
    gws.gws_sample_bwd([d3], 4)
    torch.cuda.synchronize()
    assert (synth.bits(dw2) == dw_bits).all()
    a, b = dbt3.cpu().numpy().astype(np.float64), dbt.astype(np.float64)
    _, _, asum = oracle.sample_bwd(np.ascontiguousarray(dw_bits), d.scale.cpu().numpy(), d.seed, 4)
    assert (np.abs(a - b) <= 1e-5 * np.abs(a) + 2e-6 * asum).all()


@pytest.mark.parametrize("w_is_nk", [False, True])
def test_tokens_split_into_parts(w_is_nk):
    # few tiles: the contraction over the tokens is split (2 .. 8 parts, uneven where the K-steps do not divide),
    # partial tiles go through the workspace and are added in a fixed order; dW and dL/db_t to the same bars
    run_case(1024, 256, 256, w_is_nk, 860, split=-1)                  # 1 tile, 16 K-steps: 2 parts
    run_case(2048, 512, 768, w_is_nk, 862, pad=8, split=-1)           # 6 tiles, 32 K-steps: 4 parts
    run_case(4352, 768, 256, w_is_nk, 864, row0=256, col0=512, split=-1)   # 3 tiles, 68 K-steps: 8 parts of 8 or 9
    # a workspace with room for three parts where eight were planned, and none at all
    per_part = 3 * 256 * 256 * 4
    run_case(4352, 768, 256, w_is_nk, 866, split=3 * per_part + 100)
    run_case(1024, 256, 256, w_is_nk, 868, split=0)


def test_config5_sized_weights_split_over_tokens():
    # the 2048 x 2048 weight of the 1B layer over 8192 tokens: 64 tiles in 4 parts; a row in every 256-row tile
    rng = np.random.default_rng(870)
    sel = sorted({0, 2047} | {t * 256 + int(rng.integers(0, 256)) for t in range(8)})
    run_case(8192, 2048, 2048, False, 870, rows_sel=sel, split=-1)
    d = gws.TensorDesc(rows=2048, cols=5632, seed=1)
    assert gws.gws_linear_bwd_w_workspace_bytes(d, 8192) == 0          # 176 tiles: the one-kernel form
    assert gws.gws_linear_bwd_w_workspace_bytes(gws.TensorDesc(rows=2048, cols=2048, seed=1), 8192) == 4 * 64 * 256 * 256 * 4


def test_workspace_argument_errors():
    x = torch.zeros(1024, 256, dtype=torch.bfloat16, device=DEV)
    dy = torch.zeros(1024, 256, dtype=torch.bfloat16, device=DEV)
    dw = torch.zeros(256, 256, dtype=torch.bfloat16, device=DEV)
    d = gws.TensorDesc(rows=256, cols=256, seed=1, dw=dw)
    need = gws.gws_linear_bwd_w_workspace_bytes(d, 1024)
    assert need == 2 * 256 * 256 * 4
    ws = torch.zeros(need // 4 + 4, device=DEV)
    with pytest.raises(gws.GwsError) as e:
        gws.gws_linear_bwd_w_ws(x, dy, d, 0, ws.view(torch.uint8)[4: 4 + need])      # not 16-byte aligned
    assert e.value.status == 3
    with pytest.raises(gws.GwsError) as e:
        gws.gws_linear_bwd_w_ws(x, dy, gws.TensorDesc(rows=256, cols=256, seed=1, dw=ws.view(torch.bfloat16)[:65536].view(256, 256)), 0, ws)
    assert e.value.status == 6                                                          # workspace on top of dW
    torch.cuda.synchronize()


def test_shape_and_argument_errors():
    x = torch.zeros(64, 256, dtype=torch.bfloat16, device=DEV)
    dy = torch.zeros(64, 256, dtype=torch.bfloat16, device=DEV)
    dw = torch.zeros(256, 256, dtype=torch.bfloat16, device=DEV)
    sc = torch.ones(8, 8, device=DEV)
    ok = gws.TensorDesc(rows=256, cols=256, seed=1, dw=dw, dbt=torch.zeros(8, 8, device=DEV), scale=sc)
    gws.gws_linear_bwd_w(x, dy, ok, 0)
    for bad, status in [(gws.TensorDesc(rows=128, cols=256, seed=1, dw=dw), 2),            # rows not a multiple of 256
                        (gws.TensorDesc(rows=256, cols=256, seed=1, dw=None), 1),
                        (gws.TensorDesc(rows=256, cols=256, seed=1, dw=dw, dbt=sc), 1)]:   # dbt without scale
        with pytest.raises(gws.GwsError) as e:
            gws.gws_linear_bwd_w(x, dy, bad, 0)
        assert e.value.status == status
    with pytest.raises(gws.GwsError) as e:
        gws.gws_linear_bwd_w(x[:32], dy[:32], ok, 0)                                       # M not a multiple of 64
    assert e.value.status == 2
    with pytest.raises(gws.GwsError) as e:
        gws.gws_linear_bwd_w(x, dy, gws.TensorDesc(rows=256, cols=256, seed=1, dw=x), 0)   # dW on top of X
    assert e.value.status == 6
    torch.cuda.synchronize()


def test_random_shapes():
    # seeded random weight shapes (multiples of 256) and token counts (multiples of 64: 1 .. 9 K-steps)
    rng = np.random.default_rng(1117)
    for case in range(6):
        K, N = 256 * int(rng.integers(1, 4)), 256 * int(rng.integers(1, 4))
        M = 64 * int(rng.integers(1, 10))
        run_case(M, K, N, bool(case & 1), 830 + 2 * case, pad=8 * int(rng.integers(0, 3)))
