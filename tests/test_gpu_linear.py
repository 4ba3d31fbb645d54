"""GPU parity of gws_linear_fwd / gws_linear_fwd_mode / gws_linear_fwd_ws (the sampled-weight
linear in its forms: sampling in the weight operand load, sampling kernel + plain GEMM with w_hat
in the caller's buffer or staged in a workspace) and of the plain twin gws_gemm_bf16, through the C ABI.

 - w_hat / scale written by the call: bit-exact against the oracle forward.
 - Y against the oracle's fp64 GEMM on the oracle's w_hat: |y - ref| <= 2^-8 |ref| +
   K * 2^-24 * sum|x q| (one BF16 rounding plus fp32 accumulation in any order).
 - fused Y == plain GEMM on the separately sampled w_hat, bit for bit (same GEMM code).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_11170_amd as gws
from paper_2505_11170_amd import synth
from gpu_util import DEV, ensure_built

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def bf16_val(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def check_y(y_bits, x_bits, q_bits, w_is_nk, rows_sel=None):
    K = x_bits.shape[1]
    y64, yabs, _ = oracle.linear_fwd(x_bits, q_bits, w_is_nk=w_is_nk, rows_sel=rows_sel)
    got = bf16_val(y_bits if rows_sel is None else y_bits[rows_sel])
    tol = 2.0 ** -8 * np.abs(y64) + K * 2.0 ** -24 * yabs + 1e-30
    bad = np.abs(got - y64) > tol
    assert not bad.any(), (np.argwhere(bad)[:5], got[bad][:5], y64[bad][:5])


def run_case(M, K, N, w_is_nk, fmt, bt=None, seed_id=0, step=0, rows_sel=None, ldx_pad=0, ldy_pad=0, mode=None):
    wr, wc = (N, K) if w_is_nk else (K, N)
    t = synth.make_tensor(200 + seed_id, wr, wc, bt=bt, with_grad=False)
    x_full = synth.make_activation(300 + seed_id, M, K + ldx_pad)
    x = x_full.to(DEV)[:, :K]
    w = t["w"].to(DEV)
    btd = t["bt"].to(DEV)
    seed = oracle.derive_seed(0, seed_id)
    y_store = torch.zeros(M, N + ldy_pad, dtype=torch.bfloat16, device=DEV)
    y = y_store[:, :N]
    w_hat = torch.zeros_like(w)
    nbr, nbc = synth.n_blocks(wr, wc)
    scale = torch.zeros(nbr, nbc, dtype=torch.float32, device=DEV)
    desc = gws.TensorDesc(rows=wr, cols=wc, seed=seed, w=w, w_hat=w_hat, bt=btd, scale=scale)
    if mode is None:
        gws.gws_linear_fwd(x, desc, y, fmt, step, w_is_nk=w_is_nk)
    else:
        gws.gws_linear_fwd_mode(x, desc, y, fmt, step, mode, w_is_nk=w_is_nk)
    torch.cuda.synchronize()
    # 1. sampled weight written by the call == oracle
    ref_q, ref_s = oracle.sample_fwd(synth.bits(t["w"]), t["bt"].numpy(), fmt, seed, step)
    assert (synth.bits(w_hat) == ref_q).all()
    assert (scale.cpu().numpy().view(np.uint32) == ref_s.view(np.uint32)).all()
    # 2. Y against the fp64 GEMM
    x_bits = np.ascontiguousarray(synth.bits(x_full)[:, :K])
    y_bits = np.ascontiguousarray(synth.bits(y_store)[:, :N])
    check_y(y_bits, x_bits, ref_q, w_is_nk, rows_sel)
    if ldy_pad:
        assert (synth.bits(y_store)[:, N:] == 0).all()          # padding of Y never written
    # 3. unfused path (sample kernel + plain GEMM) gives the same bits
    w_hat2 = torch.zeros_like(w)
    scale2 = torch.zeros_like(scale)
    gws.gws_sample_fwd([gws.TensorDesc(rows=wr, cols=wc, seed=seed, w=w, w_hat=w_hat2, bt=btd, scale=scale2)], fmt, step)
    y2 = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    gws.gws_gemm_bf16(x, w_hat2, y2, w_is_nk=w_is_nk)
    torch.cuda.synchronize()
    assert (synth.bits(w_hat2) == ref_q).all()
    assert (synth.bits(y2) == y_bits).all()
    # 4. without w_hat / scale outputs the result is the same
    y3 = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    gws.gws_linear_fwd(x, gws.TensorDesc(rows=wr, cols=wc, seed=seed, w=w, bt=btd), y3, fmt, step, w_is_nk=w_is_nk)
    torch.cuda.synchronize()
    assert (synth.bits(y3) == y_bits).all()
    # 5. ... and with w_hat staged in a caller's workspace (poisoned first, oversized: the tail stays as it was)
    bare = gws.TensorDesc(rows=wr, cols=wc, seed=seed, w=w, bt=btd)
    need = gws.gws_linear_fwd_workspace_bytes(bare)
    assert need == ((wr * wc * 2 + 255) // 256) * 256 + 4 * nbr * nbc
    ws = torch.full((need + 512,), 0xA5, dtype=torch.uint8, device=DEV)
    y4 = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    gws.gws_linear_fwd_ws(x, bare, y4, fmt, step, ws, w_is_nk=w_is_nk)
    torch.cuda.synchronize()
    assert (synth.bits(y4) == y_bits).all()
    assert (ws[need:] == 0xA5).all()


@pytest.mark.parametrize("w_is_nk", [False, True])
@pytest.mark.parametrize("fmt", [gws.FMT_BF16, gws.FMT_FP8_E4M3, gws.FMT_FP6_E3M2])
def test_linear_small_shapes(w_is_nk, fmt):
    run_case(128, 64, 128, w_is_nk, fmt, bt=6.0)                    # automatic choice (w_hat given: sampling kernel + GEMM)
    run_case(200, 96, 160, w_is_nk, fmt, seed_id=1)                 # two kernels; ragged M, N not a tile multiple
    run_case(37, 32, 32, w_is_nk, fmt, seed_id=2, step=3)
    run_case(300, 256, 416, w_is_nk, fmt, seed_id=3, ldx_pad=8, ldy_pad=16)
    run_case(200, 96, 160, w_is_nk, fmt, seed_id=1, mode=gws.LINEAR_IN_OPERAND)
    run_case(300, 256, 416, w_is_nk, fmt, seed_id=3, ldx_pad=8, ldy_pad=16, mode=gws.LINEAR_IN_OPERAND)
    run_case(37, 32, 32, w_is_nk, fmt, seed_id=2, step=3, mode=gws.LINEAR_TWO_KERNELS)


def test_plain_gemm_vs_fp64():
    M, K, N = 260, 192, 224
    x = synth.make_activation(1, M, K)
    w = synth.make_tensor(1, K, N, with_grad=False)["w"]
    y = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    gws.gws_gemm_bf16(x.to(DEV), w.to(DEV), y)
    torch.cuda.synchronize()
    check_y(synth.bits(y), synth.bits(x), synth.bits(w), False)
    wt = w.t().contiguous()
    y2 = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    gws.gws_gemm_bf16(x.to(DEV), wt.to(DEV), y2, w_is_nk=True)
    torch.cuda.synchronize()
    check_y(synth.bits(y2), synth.bits(x), synth.bits(wt), True)


@pytest.mark.parametrize("w_is_nk", [False, True])
def test_plain_gemm_large_tile_path(w_is_nk):
    # M, N multiples of 256 and K of 64 take the 256x256x64 kernel; 768 x 1280 = 3 x 5 tiles
    # exercises the XCD / patch tile numbering with a short last band
    M, K, N = 768, 192, 1280
    x = synth.make_activation(2, M, K)
    w = synth.make_tensor(2, K, N, with_grad=False)["w"]
    wd = (w.t().contiguous() if w_is_nk else w).to(DEV)
    y = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    gws.gws_gemm_bf16(x.to(DEV), wd, y, w_is_nk=w_is_nk)
    torch.cuda.synchronize()
    check_y(synth.bits(y), synth.bits(x), synth.bits(wd.cpu()), w_is_nk)
    # a 9 x 2 tile grid: more than one band of 8 m-tiles
    M2, K2, N2 = 2304, 64, 512
    x2 = synth.make_activation(3, M2, K2)
    w2 = synth.make_tensor(3, K2, N2, with_grad=False)["w"]
    wd2 = (w2.t().contiguous() if w_is_nk else w2).to(DEV)
    y2 = torch.zeros(M2, N2, dtype=torch.bfloat16, device=DEV)
    gws.gws_gemm_bf16(x2.to(DEV), wd2, y2, w_is_nk=w_is_nk)
    torch.cuda.synchronize()
    check_y(synth.bits(y2), synth.bits(x2), synth.bits(wd2.cpu()), w_is_nk)


@pytest.mark.parametrize("w_is_nk", [False, True])
@pytest.mark.parametrize("fmt", [gws.FMT_BF16, gws.FMT_FP8_E4M3, gws.FMT_FP6_E3M2])
def test_linear_on_the_large_tile(w_is_nk, fmt):
    # M, N multiples of 256, K of 64 and w_hat requested: sampling kernel + the 256-tile GEMM on w_hat
    run_case(512, 128, 768, w_is_nk, fmt, seed_id=7, step=2)
    run_case(256, 64, 256, w_is_nk, fmt, bt=3.0, seed_id=8)


def tile_rows(M, rng, tile=256, sub=32):
    """One row in every `tile`-row output tile, at a different 32-row MFMA sub-tile and lane row each time,
    plus the first and last row: every M-tile and, over the tiles, every wavefront quadrant is hit."""
    rows = {0, M - 1}
    for t in range(M // tile):
        rows.add(t * tile + sub * (t % (tile // sub)) + int(rng.integers(0, sub)))
    return np.array(sorted(rows))


def test_config5_fused_linear_8192x2048x5632_a_row_in_every_tile():
    M, K, N = 8192, 2048, 5632
    rows_sel = tile_rows(M, np.random.default_rng(5))
    assert len(rows_sel) >= 32 and len(set(rows_sel // 256)) == 32
    for mode in (None, gws.LINEAR_IN_OPERAND):
        run_case(M, K, N, False, gws.FMT_FP8_E4M3, bt=6.0, seed_id=5, rows_sel=rows_sel, mode=mode)


def test_config5_input_gradient_8192x5632x2048_a_row_in_every_tile():
    # dX = dY * W^T: the [K x N] weight of config 5 read as [N' x K'] = [2048 x 5632], 88 K-steps, one round of 256 tiles
    M, K, N = 8192, 5632, 2048
    dy = (synth.make_activation(51, M, K).float() * 1e-2).to(torch.bfloat16).to(DEV)
    w = synth.make_tensor(52, N, K, bt=6.0, with_grad=False)["w"].to(DEV)
    dx = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    gws.gws_gemm_bf16(dy, w, dx, w_is_nk=True)
    torch.cuda.synchronize()
    rows_sel = tile_rows(M, np.random.default_rng(51))
    check_y(synth.bits(dx), synth.bits(dy), synth.bits(w), True, rows_sel)


def test_linear_mode_errors():
    x = synth.make_activation(4, 200, 96).to(DEV)
    t = synth.make_tensor(4, 96, 160, with_grad=False)
    w, bt = t["w"].to(DEV), t["bt"].to(DEV)
    y = torch.zeros(200, 160, dtype=torch.bfloat16, device=DEV)
    full = gws.TensorDesc(rows=96, cols=160, seed=1, w=w, bt=bt, w_hat=torch.zeros_like(w), scale=torch.zeros(3, 5, device=DEV))
    bare = gws.TensorDesc(rows=96, cols=160, seed=1, w=w, bt=bt)
    with pytest.raises(gws.GwsError) as e:
        gws.gws_linear_fwd_mode(x, full, y, gws.FMT_FP8_E4M3, 0, 1)                         # a retired mode value
    assert e.value.status == 4
    with pytest.raises(gws.GwsError) as e:
        gws.gws_linear_fwd_mode(x, bare, y, gws.FMT_FP8_E4M3, 0, gws.LINEAR_TWO_KERNELS)    # nowhere to put w_hat
    assert e.value.status == 1
    with pytest.raises(gws.GwsError) as e:
        gws.gws_linear_fwd_mode(x, full, y, gws.FMT_FP8_E4M3, 0, 9)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert (synth.bits(y) == 0).all()                                                        # nothing was launched


def test_large_tile_gemm_random_shapes_and_strides():
    # the 256x256x64 tile at seeded random shapes: odd and even numbers of K-steps (1 .. 11), padded
    # leading dimensions, both weight layouts; every element against the fp64 GEMM
    rng = np.random.default_rng(2505)
    for case in range(10):
        M, N = 256 * int(rng.integers(1, 4)), 256 * int(rng.integers(1, 4))
        K = 64 * int(rng.integers(1, 12))
        w_is_nk = bool(case & 1)
        padx, padw, pady = (8 * int(rng.integers(0, 3)) for _ in range(3))
        x_full = synth.make_activation(400 + case, M, K + padx).to(DEV)
        wr, wc = (N, K) if w_is_nk else (K, N)
        w_full = synth.make_tensor(400 + case, wr, wc + padw, with_grad=False)["w"].to(DEV)
        y_full = torch.zeros(M, N + pady, dtype=torch.bfloat16, device=DEV)
        x, w, y = x_full[:, :K], w_full[:, :wc], y_full[:, :N]
        gws.gws_gemm_bf16(x, w, y, w_is_nk=w_is_nk)
        torch.cuda.synchronize()
        xb = np.ascontiguousarray(synth.bits(x_full)[:, :K])
        wb = np.ascontiguousarray(synth.bits(w_full)[:, :wc])
        check_y(np.ascontiguousarray(synth.bits(y_full)[:, :N]), xb, wb, w_is_nk)
        assert (synth.bits(y_full)[:, N:] == 0).all(), (case, "padding of Y written")


@pytest.mark.parametrize("w_is_nk", [False, True])
def test_large_tile_gemm_every_number_of_k_steps(w_is_nk):
    # the main loop is unrolled six K-steps with a tail of up to five, and the operand rings are primed for the
    # first three: 1 .. 14 K-steps take every path through prologue, loop and tail; every element against fp64
    M, N = 256, 512
    for nk in range(1, 15):
        K = 64 * nk
        x = synth.make_activation(700 + nk, M, K).to(DEV)
        wr, wc = (N, K) if w_is_nk else (K, N)
        w = synth.make_tensor(700 + nk, wr, wc, with_grad=False)["w"].to(DEV)
        y = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
        gws.gws_gemm_bf16(x, w, y, w_is_nk=w_is_nk)
        torch.cuda.synchronize()
        check_y(synth.bits(y), synth.bits(x), synth.bits(w), w_is_nk)


def run_next_case(M, K, N, w_is_nk, next_rows, next_cols, fmt, idx, step=3, next_pad=0, rows_sel=None):
    """gws_gemm_bf16_sample_next: Y against the fp64 GEMM, the riding forward pass against the oracle."""
    x = synth.make_activation(500 + idx, M, K).to(DEV)
    wr, wc = (N, K) if w_is_nk else (K, N)
    w = synth.make_tensor(500 + idx, wr, wc, with_grad=False)["w"].to(DEV)
    y = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    t = synth.make_tensor(600 + idx, next_rows, next_cols, ld=next_cols + next_pad, with_grad=False)
    nw, nbt = t["w"].to(DEV), t["bt"].to(DEV)
    n_hat = nw.clone()                                     # padding columns must keep these bytes
    nbr, nbc = synth.n_blocks(next_rows, next_cols)
    n_scale = torch.full((nbr, nbc), float("nan"), device=DEV)
    seed = oracle.derive_seed(7, idx)
    nxt = gws.TensorDesc(rows=next_rows, cols=next_cols, ld=next_cols + next_pad, seed=seed, w=nw, w_hat=n_hat, bt=nbt, scale=n_scale)
    gws.gws_gemm_bf16_sample_next(x, w, y, nxt, fmt, step, w_is_nk=w_is_nk)
    torch.cuda.synchronize()
    check_y(synth.bits(y), synth.bits(x), synth.bits(w), w_is_nk, rows_sel)
    ref_q, ref_s = oracle.sample_fwd(synth.bits(t["w"]), t["bt"].numpy(), fmt, seed, step, cols=next_cols)
    assert (synth.bits(n_hat) == ref_q).all(), ("w_hat of the next weight", idx)
    assert (n_scale.cpu().numpy().view(np.uint32) == ref_s.view(np.uint32)).all(), ("scale of the next weight", idx)
    return y


@pytest.mark.parametrize("fmt", [gws.FMT_BF16, gws.FMT_FP8_E4M3, gws.FMT_FP6_E3M2])
def test_gemm_with_the_next_weight_sampled_alongside(fmt):
    run_next_case(768, 192, 1280, False, 128, 320, fmt, 0)                   # 15 tiles: the sampling rides in the same launch
    run_next_case(512, 128, 512, True, 256, 1024, fmt, 1, next_pad=8)        # [N x K] weight, padded next weight
    run_next_case(768, 192, 1280, False, 96, 300, fmt, 2, next_pad=4)        # ragged next weight: separate launch
    run_next_case(200, 96, 160, False, 128, 320, fmt, 3)                     # GEMM not on the large tile: separate launch
    run_next_case(256, 64, 256, False, 4096, 4096, fmt, 4)                   # sampling far longer than the GEMM: separate launch


def test_gemm_next_without_idle_compute_units_and_without_next():
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert cus % 16 == 0
    M, N = 256 * 16, 256 * (cus // 16)                                       # exactly one tile per compute unit
    y = run_next_case(M, 64, N, False, 128, 320, gws.FMT_FP8_E4M3, 5, rows_sel=np.array([0, 255, 256, M - 1]))
    # next = None is the plain GEMM
    x = synth.make_activation(505, M, 64).to(DEV)
    w = synth.make_tensor(505, 64, N, with_grad=False)["w"].to(DEV)
    y2 = torch.zeros_like(y)
    gws.gws_gemm_bf16_sample_next(x, w, y2, None, gws.FMT_FP8_E4M3, 0)
    torch.cuda.synchronize()
    assert (synth.bits(y2) == synth.bits(y)).all()


def test_config5_gemm_with_the_next_weight_sampled_alongside():
    rows_sel = tile_rows(8192, np.random.default_rng(6))
    run_next_case(8192, 2048, 5632, False, 2048, 5632, gws.FMT_FP8_E4M3, 6, rows_sel=rows_sel)   # too much to ride: two launches
    run_next_case(8192, 2048, 5632, False, 2048, 2048, gws.FMT_FP8_E4M3, 7, rows_sel=rows_sel)   # rides beside the last round of tiles


def run_next_list(M, K, N, next_shapes, fmt, idx, step=5, rows_sel=None):
    """gws_gemm_bf16_sample_next_n: Y against the fp64 GEMM, every listed weight against the oracle's forward pass."""
    x = synth.make_activation(700 + idx, M, K).to(DEV)
    w = synth.make_tensor(700 + idx, K, N, with_grad=False)["w"].to(DEV)
    y = torch.zeros(M, N, dtype=torch.bfloat16, device=DEV)
    descs, host = [], []
    for k, (r, c) in enumerate(next_shapes):
        ld = (c + 7) // 8 * 8
        t = synth.make_tensor(720 + 10 * idx + k, r, c, ld=ld, with_grad=False)
        nw = t["w"].to(DEV)
        nbr, nbc = synth.n_blocks(r, c)
        descs.append(gws.TensorDesc(rows=r, cols=c, ld=ld, seed=oracle.derive_seed(9, 10 * idx + k), w=nw, w_hat=nw.clone(),
                                    bt=t["bt"].to(DEV), scale=torch.full((nbr, nbc), float("nan"), device=DEV)))
        host.append(t)
    gws.gws_gemm_bf16_sample_next_n(x, w, y, descs, fmt, step)
    torch.cuda.synchronize()
    check_y(synth.bits(y), synth.bits(x), synth.bits(w), False, rows_sel)
    for d, t in zip(descs, host):
        ref_q, ref_s = oracle.sample_fwd(synth.bits(t["w"]), t["bt"].numpy(), fmt, d.seed, step, cols=d.cols)
        assert (synth.bits(d.w_hat) == ref_q).all(), ("w_hat", idx, d.rows, d.cols)
        assert (d.scale.cpu().numpy().view(np.uint32) == ref_s.view(np.uint32)).all(), ("scale", idx, d.rows, d.cols)


@pytest.mark.parametrize("fmt", [gws.FMT_BF16, gws.FMT_FP8_E4M3, gws.FMT_FP6_E3M2])
def test_gemm_with_several_next_weights_sampled_alongside(fmt):
    run_next_list(768, 192, 1280, [(128, 512), (64, 256), (96, 768)], fmt, 0)           # all three ride (whole 32 x 256 tiles)
    run_next_list(768, 192, 1280, [(128, 512), (96, 300)], fmt, 1)                       # the ragged one: separate launch
    run_next_list(768, 192, 1280, [(32, 256)] * 5 + [(64, 512)], fmt, 2)                 # more than ride at once: the rest after the GEMM
    run_next_list(768, 192, 1280, [(96, 320), (128, 512)], fmt, 3)                       # first not of whole 32 x 256 tiles: rides alone
    run_next_list(200, 96, 160, [(128, 512), (64, 256)], fmt, 4)                         # GEMM not on the large tile: all separate
    run_next_list(768, 192, 1280, [(256, 512), (0, 256), (64, 256)], fmt, 5)             # an empty weight in the list
    run_next_list(256, 64, 256, [(2048, 2048), (1024, 1024)], fmt, 6)                    # too much to ride beside one short tile


def test_forced_riding_gives_the_same_bytes_for_both_riding_loops():
    # include/gws_bench.h, gws_gemm_bf16_ride_probe: riders alone (no GEMM) and beside a GEMM, both riding loops
    fmt, step = gws.FMT_FP8_E4M3, 8
    t = synth.make_tensor(790, 512, 1280, with_grad=False)
    seed = oracle.derive_seed(3, 790)
    ref_q, ref_s = oracle.sample_fwd(synth.bits(t["w"]), t["bt"].numpy(), fmt, seed, step)
    nw, nbt = t["w"].to(DEV), t["bt"].to(DEV)
    x = synth.make_activation(791, 512, 128).to(DEV)
    w = synth.make_tensor(791, 128, 768, with_grad=False)["w"].to(DEV)
    for rider in (0, 1):
        for with_gemm in (False, True):
            for extra in (1, 7, 64):
                d = gws.TensorDesc(rows=512, cols=1280, seed=seed, w=nw, w_hat=torch.zeros_like(nw), bt=nbt,
                                   scale=torch.zeros(16, 40, device=DEV))
                y = torch.zeros(512, 768, dtype=torch.bfloat16, device=DEV)
                if with_gemm:
                    gws.gws_gemm_bf16_ride_probe(x, w, y, d, fmt, step, extra, rider)
                else:
                    gws.gws_gemm_bf16_ride_probe(None, None, None, d, fmt, step, extra, rider)
                torch.cuda.synchronize()
                assert (synth.bits(d.w_hat) == ref_q).all(), (rider, with_gemm, extra)
                assert (d.scale.cpu().numpy().view(np.uint32) == ref_s.view(np.uint32)).all()
                if with_gemm:
                    check_y(synth.bits(y), synth.bits(x), synth.bits(w), False)
