"""GPU parity of the comparison noise bases (paper Sec. 4: BF16 U(-0.5, 0.5), Box-Muller round(N(0,1)/2)) behind
gws_sample_fwd_basis / gws_sample_bwd_basis / gws_noise_basis, through the C ABI, against the oracle.

Bit-exact: R itself, the sampled and cast weights, scale, dW.  dL/db_t within 1e-5 relative (+ the rounding floor).
The Box-Muller basis decides an integer in floating point; both sides evaluate the same fp32 sequence, and the
full-size cases below put 10^9 elements through it (a square root off by one ulp would show as a few mismatches)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_11170_amd as gws
from paper_2505_11170_amd import synth
from gpu_util import DEV, assert_dbt_close, ensure_built

pytestmark = pytest.mark.gpu

BASES = {"uniform": (gws.BASIS_UNIFORM_BF16, oracle.BASIS_UNIFORM), "box_muller": (gws.BASIS_BOX_MULLER, oracle.BASIS_BOX_MULLER)}
FMTS = [gws.FMT_BF16, gws.FMT_FP8_E4M3, gws.FMT_FP6_E3M2]


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def bf16_f32(bits):
    return (np.ascontiguousarray(bits).astype(np.uint32) << 16).view(np.float32)


@pytest.mark.parametrize("name", list(BASES))
def test_noise_of_a_basis_matches_the_oracle(name):
    gb, ob = BASES[name]
    for rows, cols, row0, col0, seed, step in [(64, 256, 0, 0, 1, 0), (33, 40, 96, 64, oracle.derive_seed(5, 5), 2 ** 40 + 3),
                                                (4096, 4096, 0, 0, oracle.derive_seed(8, 1), 7)]:
        out = torch.zeros(rows, cols, dtype=torch.bfloat16, device=DEV)
        gws.gws_noise_basis(out, rows, cols, seed, step, gb, row0=row0, col0=col0)
        torch.cuda.synchronize()
        ref = oracle.noise_basis(rows, cols, seed, step, ob, row0=row0, col0=col0)
        got = bf16_f32(synth.bits(out))
        assert (got.view(np.uint32) == ref.view(np.uint32)).all(), (name, rows, cols)   # sign of a zero included


def run_fwd_bwd(shapes, gb, ob, fmt, step, bt=None, pads=None, copy_dw=True):
    descs, host = [], []
    for i, (r, c) in enumerate(shapes):
        ld = c + (pads[i] if pads else 0)
        t = synth.make_tensor(1200 + i, r, c, bt=bt, ld=(ld + 7) // 8 * 8)
        nbr, nbc = synth.n_blocks(r, c)
        w, g = t["w"].to(DEV), t["g"].to(DEV)
        d = gws.TensorDesc(rows=r, cols=c, ld=t["w"].stride(0), seed=oracle.derive_seed(4, i), w=w, w_hat=w.clone(),
                           bt=t["bt"].to(DEV), scale=torch.full((nbr, nbc), float("nan"), device=DEV), g=g,
                           dw=(torch.zeros_like(g) if copy_dw else g), dbt=torch.full((nbr, nbc), float("nan"), device=DEV))
        descs.append(d)
        host.append(t)
    gws.gws_sample_fwd_basis(descs, gb, fmt, step)
    gws.gws_sample_bwd_basis(descs, gb, step)
    torch.cuda.synchronize()
    for d, t in zip(descs, host):
        ref_q, ref_s = oracle.sample_fwd(synth.bits(t["w"]), t["bt"].numpy(), fmt, d.seed, step, cols=d.cols, basis=ob)
        assert (d.scale.cpu().numpy().view(np.uint32) == ref_s.view(np.uint32)).all(), (d.rows, d.cols)
        got = synth.bits(d.w_hat)
        bad = np.argwhere(got != ref_q)
        assert len(bad) == 0, (d.rows, d.cols, [(int(i), int(j), hex(got[i, j]), hex(ref_q[i, j])) for i, j in bad[:6]])
        ref_dw, ref_dbt, asum = oracle.sample_bwd(synth.bits(t["g"]), ref_s, d.seed, step, cols=d.cols, basis=ob)
        if copy_dw:
            assert (synth.bits(d.dw)[:, :d.cols] == ref_dw[:, :d.cols]).all()
            assert (synth.bits(d.dw)[:, d.cols:] == 0).all()                      # padding never written
        assert_dbt_close(d.dbt.cpu().numpy(), ref_dbt, asum, (d.rows, d.cols))


@pytest.mark.parametrize("name", list(BASES))
@pytest.mark.parametrize("fmt", FMTS)
def test_forward_backward_ragged_and_full_shapes(name, fmt):
    gb, ob = BASES[name]
    run_fwd_bwd([(768, 768), (96, 320), (40, 50), (33, 257), (1, 1), (64, 8)], gb, ob, fmt, step=5, pads=[0, 8, 6, 7, 7, 0])
    run_fwd_bwd([(256, 512)], gb, ob, fmt, step=1, bt=2.0)           # coarse noise: the cast saturates in places
    run_fwd_bwd([(128, 256)], gb, ob, fmt, step=1, bt=9.0, copy_dw=False)


@pytest.mark.parametrize("name", list(BASES))
def test_config2_gpt2_124m_with_a_comparison_basis(name):
    gb, ob = BASES[name]
    shapes = [(s.rows, s.cols) for s in synth.gpt2_124m_shapes()]
    run_fwd_bwd(shapes, gb, ob, gws.FMT_FP8_E4M3, step=2, copy_dw=False)


def test_config3_llama_1b_box_muller_forward_every_element():
    # 968 884 224 rounded normals decided in fp32 on both sides
    gb, ob = BASES["box_muller"]
    shapes = synth.llama_1b_shapes()
    descs = []
    for i, sh in enumerate(shapes):
        t = synth.make_tensor(i, sh.rows, sh.cols, device=DEV, with_grad=False)
        nbr, nbc = synth.n_blocks(sh.rows, sh.cols)
        descs.append(gws.TensorDesc(rows=sh.rows, cols=sh.cols, seed=gws.gws_derive_seed(0, i), w=t["w"],
                                    w_hat=torch.zeros_like(t["w"]), bt=t["bt"], scale=torch.zeros(nbr, nbc, device=DEV)))
    gws.gws_sample_fwd_basis(gws.pack(descs), gb, gws.FMT_FP8_E4M3, 0)
    torch.cuda.synchronize()
    for d, sh in zip(descs, shapes):
        ref_q, ref_s = oracle.sample_fwd(synth.bits(d.w), d.bt.cpu().numpy(), oracle.FMT_FP8_E4M3, d.seed, 0, basis=ob)
        assert (d.scale.cpu().numpy().view(np.uint32) == ref_s.view(np.uint32)).all(), sh
        assert (synth.bits(d.w_hat) == ref_q).all(), sh
        d.w_hat = None


def test_basis_argument_rules():
    t = synth.make_tensor(1, 64, 64)
    d = gws.TensorDesc(rows=64, cols=64, seed=1, w=t["w"].to(DEV), w_hat=torch.zeros(64, 64, dtype=torch.bfloat16, device=DEV),
                       bt=t["bt"].to(DEV), scale=torch.zeros(2, 2, device=DEV), g=t["g"].to(DEV), dbt=torch.zeros(2, 2, device=DEV))
    for bad in (3, -1):
        with pytest.raises(gws.GwsError) as e:
            gws.gws_sample_fwd_basis([d], bad, gws.FMT_BF16, 0)
        assert e.value.status == 4
        with pytest.raises(gws.GwsError) as e:
            gws.gws_sample_bwd_basis([d], bad, 0)
        assert e.value.status == 4
    # basis 0 is the method's own: the same bytes as gws_sample_fwd
    gws.gws_sample_fwd_basis([d], gws.BASIS_BITS, gws.FMT_FP8_E4M3, 3)
    a = d.w_hat.clone()
    gws.gws_sample_fwd([d], gws.FMT_FP8_E4M3, 3)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), d.w_hat.view(torch.int16))
    out = torch.zeros(8, 12, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(gws.GwsError) as e:
        gws.gws_noise_basis(out, 8, 12, 1, 0, gws.BASIS_UNIFORM_BF16)              # cols not a multiple of 8
    assert e.value.status == 2
