"""GPU parity of gws_sample_fwd_mx (element codes + E8M0 block scales) against the CPU oracle,
through the C ABI.  Everything here is bytes: bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_11170_amd as gws
from paper_2505_11170_amd import synth
from gpu_util import DEV, ensure_built

pytestmark = pytest.mark.gpu

MX_FMTS = [gws.FMT_FP8_E4M3, gws.FMT_FP6_E3M2]


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def row_stride(cols, fmt, pad):
    nb = oracle.mx_row_bytes(cols, fmt)
    mult = 8 if fmt == gws.FMT_FP8_E4M3 else 2
    return (nb + mult - 1) // mult * mult + pad * mult


def run_mx(items, fmt, step, pad=0):
    descs, outs, keep = [], [], []
    for it in items:
        w, bt = it["w"].to(DEV), it["bt"].to(DEV)
        nbr, nbc = synth.n_blocks(it["rows"], it["cols"])
        ldc = row_stride(it["cols"], fmt, pad)
        codes = torch.full((max(it["rows"], 1), max(ldc, 1)), 0xAA, dtype=torch.uint8, device=DEV)
        xscale = torch.full((nbr, nbc), 0xEE, dtype=torch.uint8, device=DEV)
        scale = torch.full((nbr, nbc), float("nan"), device=DEV)
        descs.append(gws.TensorDesc(rows=it["rows"], cols=it["cols"], seed=it["seed"], w=w, bt=bt, scale=scale,
                                    ld=w.stride(0) if w.numel() else it["cols"],
                                    row0=it.get("row0", 0), col0=it.get("col0", 0)))
        outs.append(gws.MxOut(codes=codes, xscale=xscale, ldc=ldc))
        keep.append((codes, xscale, scale, ldc))
    gws.gws_sample_fwd_mx(descs, outs, fmt, step)
    torch.cuda.synchronize()
    return [(k[0].cpu().numpy(), k[1].cpu().numpy(), k[2].cpu().numpy(), k[3]) for k in keep]


def check_mx(items, fmt, step, pad=0):
    res = run_mx(items, fmt, step, pad)
    for it, (codes, xscale, scale, ldc) in zip(items, res):
        if it["rows"] == 0 or it["cols"] == 0:
            continue
        ref_c, ref_x, ref_s = oracle.sample_fwd_mx(synth.bits(it["w"]), it["bt"].numpy(), fmt, it["seed"], step,
                                                   cols=it["cols"], row0=it.get("row0", 0), col0=it.get("col0", 0), ldc=ldc)
        what = (it["rows"], it["cols"], fmt)
        assert np.array_equal(scale.view(np.uint32), ref_s.view(np.uint32)), ("scale",) + what
        assert np.array_equal(xscale, ref_x), ("xscale",) + what
        bad = np.argwhere(codes[:it["rows"]] != ref_c)     # includes the 0xAA bytes past each row's data
        assert len(bad) == 0, ("codes",) + what + (bad[:5],)


def make_items(shapes, base, bt=None, user_seed=0):
    items = []
    for i, (r, c) in enumerate(shapes):
        t = synth.make_tensor(base + i, r, c, bt=bt, ld=(c + 7) // 8 * 8, with_grad=False)
        items.append(dict(w=t["w"], bt=t["bt"], rows=r, cols=c, seed=oracle.derive_seed(user_seed, base + i)))
    return items


@pytest.mark.parametrize("fmt", MX_FMTS)
def test_config1_shape_and_a_batch(fmt):
    check_mx(make_items([(768, 768)], 400, bt=6.0), fmt, 0)
    check_mx(make_items([(768, 2304), (96, 320), (3072, 768), (32, 32), (0, 64), (256, 64)], 410), fmt, 5)


@pytest.mark.parametrize("fmt", MX_FMTS)
def test_ragged_shapes_and_padded_rows(fmt):
    shapes = [(40, 50), (33, 257), (1, 1), (31, 7), (65, 300), (100, 36)]
    check_mx(make_items(shapes, 420), fmt, 1, pad=0)
    check_mx(make_items(shapes, 420), fmt, 1, pad=3)


@pytest.mark.parametrize("fmt", MX_FMTS)
def test_low_bitwidths_reach_saturation_and_the_arithmetic_encoder(fmt):
    # b_t <= 2 lets w + 2s exceed the largest finite code: the saturating path must agree too
    for bt in (1.0, 1.5, 2.0, 3.0):
        check_mx(make_items([(128, 256), (64, 96)], 430, bt=bt), fmt, 2)


@pytest.mark.parametrize("fmt", MX_FMTS)
def test_edge_values_and_zero_blocks(fmt):
    r, c = 64, 128
    t = synth.make_tensor(440, r, c, with_grad=False)
    w = t["w"].clone()
    w[:32, :32] = 0.0                          # an all-zero block
    w[0, 0] = -0.0
    w[:32, 32:64] = 2.0 ** -60                 # a tiny block: its scale exponent is far below 127
    w[32:, 64:96] *= 2.0 ** 30                 # and a huge one
    w[40, 70] = -1.0e12
    item = dict(w=w, bt=t["bt"], rows=r, cols=c, seed=7)
    check_mx([item], fmt, 3)


@pytest.mark.parametrize("fmt", MX_FMTS)
def test_config2_all_48_weights_in_one_launch(fmt):
    # the launch configuration bench.py times; the oracle checks one tensor of each shape in full
    shapes = [(s.rows, s.cols) for s in synth.gpt2_124m_shapes()]
    items = make_items(shapes, 0)
    res = run_mx(items, fmt, 1)
    seen = set()
    for it, (codes, xscale, scale, ldc) in zip(items, res):
        if (it["rows"], it["cols"]) in seen:
            continue
        seen.add((it["rows"], it["cols"]))
        ref_c, ref_x, ref_s = oracle.sample_fwd_mx(synth.bits(it["w"]), it["bt"].numpy(), fmt, it["seed"], 1, ldc=ldc)
        assert np.array_equal(scale.view(np.uint32), ref_s.view(np.uint32))
        assert np.array_equal(xscale, ref_x) and np.array_equal(codes, ref_c), (it["rows"], it["cols"])
    assert len(seen) == 4


def test_shard_origin_reproduces_the_unsharded_codes():
    r, c = 128, 256
    item = make_items([(r, c)], 450)[0]
    full = run_mx([item], gws.FMT_FP8_E4M3, 4)[0]
    shard = dict(w=item["w"][64:, 128:].contiguous(), bt=item["bt"][2:, 4:].contiguous(), rows=64, cols=128,
                 seed=item["seed"], row0=64, col0=128)
    part = run_mx([shard], gws.FMT_FP8_E4M3, 4)[0]
    assert np.array_equal(part[0][:, :128], full[0][64:, 128:256])
    assert np.array_equal(part[1], full[1][2:, 4:])


def test_argument_errors():
    t = synth.make_tensor(460, 64, 64, with_grad=False)
    w, bt = t["w"].to(DEV), t["bt"].to(DEV)
    d = gws.TensorDesc(rows=64, cols=64, seed=1, w=w, bt=bt, scale=torch.empty_like(bt))
    codes = torch.empty(64, 64, dtype=torch.uint8, device=DEV)
    xs = torch.empty(2, 2, dtype=torch.uint8, device=DEV)
    with pytest.raises(gws.GwsError) as e:
        gws.gws_sample_fwd_mx([d], [gws.MxOut(codes, xs)], gws.FMT_BF16, 0)       # no MX form of BF16
    assert e.value.status == 4
    with pytest.raises(gws.GwsError) as e:
        gws.gws_sample_fwd_mx([d], [gws.MxOut(codes, xs, ldc=60)], gws.FMT_FP8_E4M3, 0)   # row stride too small
    assert e.value.status == 2
    with pytest.raises(gws.GwsError) as e:
        gws.gws_sample_fwd_mx([d], [gws.MxOut(codes, None)], gws.FMT_FP8_E4M3, 0)
    assert e.value.status == 1
    with pytest.raises(gws.GwsError) as e:
        gws.gws_sample_fwd_mx([d], [gws.MxOut(codes.view(-1)[1:4033].view(63, 64), xs, ldc=64)], gws.FMT_FP8_E4M3, 0)
    assert e.value.status == 3
    torch.cuda.synchronize()


@pytest.mark.parametrize("fmt", MX_FMTS)
def test_random_mix_of_many_small_and_ragged_tensors(fmt):
    rng = np.random.default_rng(40 + fmt)
    shapes = [(int(rng.integers(1, 150)), int(rng.integers(1, 1100))) for _ in range(64)]
    shapes[3] = (0, 17)
    shapes[9] = (32, 256)
    check_mx(make_items(shapes, 2000 + 100 * fmt, user_seed=fmt), fmt, 6, pad=1)
