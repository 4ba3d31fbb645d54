"""GPU parity at the full sizes of the large configurations, through the C ABI, in the
launch configuration bench.py times (every weight of the model in one descriptor list).

config 3: all 154 linear weights of the ~1B Llama2-style decoder (968 884 224 params),
          fwd + bwd, every element against the oracle.
config 4: precision sweep {4,...,9, U[4,9]} x {FP6-E3M2, FP8-E4M3, BF16}: every element of
          one decoder layer per cell, plus sampled 32x32 blocks of the full model per cell
          (the oracle recomputes a block on its own from (row0, col0)).
Inputs are generated on the GPU from seeded generators and copied to the host for the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_11170_amd as gws
from paper_2505_11170_amd import synth
from gpu_util import CANCELLATION_SHARE, DEV, assert_dbt_close, ensure_built

pytestmark = pytest.mark.gpu

FMTS = {"fp6_e3m2": gws.FMT_FP6_E3M2, "fp8_e4m3": gws.FMT_FP8_E4M3, "bf16": gws.FMT_BF16}
PRECISIONS = [4.0, 5.0, 6.0, 7.0, 8.0, 9.0, None]      # None = heterogeneous U[4, 9] per block


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def device_set(shapes, bt=None, with_grad=True, copy_dw=True):
    descs = []
    for i, sh in enumerate(shapes):
        t = synth.make_tensor(i, sh.rows, sh.cols, bt=bt, device=DEV, with_grad=with_grad)
        nbr, nbc = synth.n_blocks(sh.rows, sh.cols)
        descs.append(gws.TensorDesc(
            rows=sh.rows, cols=sh.cols, seed=gws.gws_derive_seed(0, i), w=t["w"], w_hat=torch.zeros_like(t["w"]),
            bt=t["bt"], scale=torch.zeros(nbr, nbc, device=DEV), g=t["g"],
            dw=(torch.zeros_like(t["g"]) if (with_grad and copy_dw) else t["g"]),
            dbt=torch.zeros(nbr, nbc, device=DEV)))
    return descs


def test_config3_llama_1b_every_element_fwd_bwd():
    shapes = synth.llama_1b_shapes()
    assert len(shapes) == 154 and sum(s.rows * s.cols for s in shapes) == 968_884_224
    descs = device_set(shapes)
    pk = gws.pack(descs)
    step = 0
    gws.gws_sample_fwd(pk, gws.FMT_FP8_E4M3, step)
    gws.gws_sample_bwd(pk, step)
    torch.cuda.synchronize()
    needed = 0
    for i, d in enumerate(descs):
        ref_q, ref_s = oracle.sample_fwd(synth.bits(d.w), d.bt.cpu().numpy(), oracle.FMT_FP8_E4M3, d.seed, step)
        assert (d.scale.cpu().numpy().view(np.uint32) == ref_s.view(np.uint32)).all(), shapes[i]
        assert (synth.bits(d.w_hat) == ref_q).all(), shapes[i]
        ref_dw, ref_dbt, asum = oracle.sample_bwd(synth.bits(d.g), ref_s, d.seed, step)
        assert (synth.bits(d.dw) == ref_dw).all(), shapes[i]
        needed += assert_dbt_close(d.dbt.cpu().numpy(), ref_dbt, asum, shapes[i])
        d.w_hat = d.dw = None   # free as we go
    print(f"config 3: blocks needing the cancellation term of the db_t tolerance: {needed} of 946176")
    # the benchmark spec's tolerance is the relative term; the additive floor may only be what decides for the few blocks
    # whose +- terms cancel to below 1e-5 of their absolute sum
    assert needed <= CANCELLATION_SHARE * 946176


@pytest.mark.parametrize("fmt_name", list(FMTS))
def test_config4_precision_sweep(fmt_name):
    fmt = FMTS[fmt_name]
    shapes = synth.llama_1b_shapes()
    layer = shapes[:7]
    rng = np.random.default_rng(4)
    for bt in PRECISIONS:
        # (a) one decoder layer, every element
        descs = device_set(layer, bt=bt, with_grad=(fmt == gws.FMT_BF16))
        gws.gws_sample_fwd(descs, fmt, 1)
        if fmt == gws.FMT_BF16:
            gws.gws_sample_bwd(descs, 1)
        torch.cuda.synchronize()
        for d, sh in zip(descs, layer):
            ref_q, ref_s = oracle.sample_fwd(synth.bits(d.w), d.bt.cpu().numpy(), fmt, d.seed, 1)
            assert (d.scale.cpu().numpy().view(np.uint32) == ref_s.view(np.uint32)).all(), (sh, bt)
            assert (synth.bits(d.w_hat) == ref_q).all(), (sh, bt)
            if fmt == gws.FMT_BF16:      # backward does not depend on the target format
                ref_dw, ref_dbt, asum = oracle.sample_bwd(synth.bits(d.g), ref_s, d.seed, 1)
                assert (synth.bits(d.dw) == ref_dw).all()
                assert_dbt_close(d.dbt.cpu().numpy(), ref_dbt, asum, (sh, bt))
        del descs
    # (b) the full model in one descriptor list, sampled blocks, in every one of the seven precision settings
    # (the weights are the same in all of them: only the b_t tables change between the launches)
    descs = device_set(shapes, bt=None, with_grad=False)
    het = [d.bt.clone() for d in descs]
    pk = gws.pack(descs)
    for bt in PRECISIONS:
        for d, h in zip(descs, het):
            d.bt.copy_(h) if bt is None else d.bt.fill_(bt)
        gws.gws_sample_fwd(pk, fmt, 2)
        torch.cuda.synchronize()
        for _ in range(64):
            ti = int(rng.integers(0, len(descs)))
            d = descs[ti]
            bi, bj = int(rng.integers(0, d.rows // 32)), int(rng.integers(0, d.cols // 32))
            wb = synth.bits(d.w[bi * 32:bi * 32 + 32, bj * 32:bj * 32 + 32].contiguous())
            btb = d.bt[bi:bi + 1, bj:bj + 1].cpu().numpy()
            ref_q, ref_s = oracle.sample_fwd(wb, btb, fmt, d.seed, 2, row0=bi * 32, col0=bj * 32)
            got = synth.bits(d.w_hat[bi * 32:bi * 32 + 32, bj * 32:bj * 32 + 32].contiguous())
            assert (got == ref_q).all(), (ti, bi, bj, bt)
            assert d.scale[bi, bj].item() == ref_s[0, 0]
    del descs, pk, het
    torch.cuda.empty_cache()


def test_one_tensor_beyond_4_gib_matches_its_shards_and_the_oracle():
    # a ragged tensor of 2.29e9 elements (4.6 GB per buffer): byte offsets pass 2^32 inside one tensor.
    # (a) every element equals what four row shards of about 1.15 GB each give through their origins,
    # (b) sampled blocks, the last (ragged) block row and column among them, equal the oracle's.
    rows, cols, ld = 40_011, 57_350, 57_352
    assert rows * ld * 2 > 2 ** 32
    step, fmt = 11, gws.FMT_FP8_E4M3
    t = synth.make_tensor(90, rows, cols, device=DEV, ld=ld)
    seed = gws.gws_derive_seed(3, 90)
    nbr, nbc = synth.n_blocks(rows, cols)
    w, g, bt = t["w"], t["g"], t["bt"]

    def run(r0, r1, w_hat, scale, dw, dbt):
        b0, b1 = r0 // 32, (r1 + 31) // 32
        d = gws.TensorDesc(rows=r1 - r0, cols=cols, ld=ld, seed=seed, row0=r0, w=w[r0:r1], w_hat=w_hat[r0:r1],
                           bt=bt[b0:b1], scale=scale[b0:b1], g=g[r0:r1], dw=dw[r0:r1], dbt=dbt[b0:b1])
        gws.gws_sample_fwd([d], fmt, step)
        gws.gws_sample_bwd([d], step)

    def outputs():
        return (w.clone(), torch.zeros(nbr, nbc, device=DEV), torch.zeros_like(g), torch.zeros(nbr, nbc, device=DEV))

    whole = outputs()
    run(0, rows, *whole)
    torch.cuda.synchronize()
    parts = outputs()
    cuts = [0, 10_016, 20_000, 30_016, rows]
    for r0, r1 in zip(cuts[:-1], cuts[1:]):
        run(r0, r1, *parts)
    torch.cuda.synchronize()
    names = ("w_hat", "scale", "dw", "db_t")
    for name, a, b in zip(names, whole, parts):
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a.view(torch.int32),
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b.view(torch.int32)), name
    del parts
    w_hat, scale, dw, dbt = whole
    assert torch.equal(w_hat[:, cols:].view(torch.int16), w[:, cols:].view(torch.int16)), "padding written"
    assert torch.equal(dw[:, :cols].view(torch.int16), g[:, :cols].view(torch.int16))
    assert not torch.equal(w_hat[-64:, :cols].view(torch.int16), w[-64:, :cols].view(torch.int16))

    rng = np.random.default_rng(90)
    picks = [(nbr - 1, nbc - 1), (nbr - 1, 0), (0, nbc - 1), (nbr - 2, nbc - 2), (0, 0)]
    picks += [(int(rng.integers(0, nbr)), int(rng.integers(0, nbc))) for _ in range(30)]
    first_beyond = 2 ** 32 // (2 * ld * 32) + 1                            # block rows whose bytes lie past 2^32
    picks += [(int(rng.integers(first_beyond, nbr)), int(rng.integers(0, nbc))) for _ in range(29)]
    beyond = 0
    for bi, bj in picks:
        r0, c0 = bi * 32, bj * 32
        nr, nc = min(32, rows - r0), min(32, cols - c0)
        beyond += (r0 * ld + c0) * 2 >= 2 ** 32
        wb = synth.bits(w[r0:r0 + nr, c0:c0 + 32].contiguous())            # 32 wide: ld stays a multiple of 8
        btb = bt[bi:bi + 1, bj:bj + 1].cpu().numpy()
        ref_q, ref_s = oracle.sample_fwd(wb, btb, fmt, seed, step, cols=nc, row0=r0, col0=c0)
        got = synth.bits(w_hat[r0:r0 + nr, c0:c0 + 32].contiguous())
        assert (got[:, :nc] == ref_q[:, :nc]).all(), (bi, bj)
        assert scale[bi, bj].item() == ref_s[0, 0], (bi, bj)
        gb = synth.bits(g[r0:r0 + nr, c0:c0 + 32].contiguous())
        _, ref_dbt, asum = oracle.sample_bwd(gb, ref_s, seed, step, cols=nc, row0=r0, col0=c0)
        assert_dbt_close(dbt[bi:bi + 1, bj:bj + 1].cpu().numpy(), ref_dbt, asum, (bi, bj))
    assert beyond >= 29
