"""Every finite BF16 pattern through the cast of the forward pass (paper Sec. 3.3), on the GPU, against the oracle.

The synthetic weights of the other parity tests (N(0, 0.02) plus a few edge values) reach only a small part of the
BF16 patterns relative to a block's scale.  Here a tensor is built whose 32x32 blocks each hold a planted maximum
`a` and a slice of ALL BF16 patterns of magnitude <= a (both signs, zeros and subnormals included), for several
maxima (different mantissas, a tiny and a huge binade) and four bitwidths chosen so that every branch of the
kernel's cast is taken:
  b_t = 60  the noise is below half an ulp of everything but the smallest values: the cast sees the patterns themselves
  b_t = 6   ordinary noise; the block cannot overflow, so FP8-E4M3 goes through the hardware converters
  b_t = 2   |R s| reaches the block maximum: for maxima above 1.75 * 2^Ea the block may overflow and FP8-E4M3
            takes the arithmetic cast
  b_t = 1   |R s| reaches twice the block maximum: values beyond the format's largest code occur (saturation)
FP8-E4M3 and FP6-E3M2, both as the BF16 container (gws_sample_fwd) and as MX element codes + E8M0 block scales
(gws_sample_fwd_mx), element by element against oracle.sample_fwd / oracle.sample_fwd_mx; a ragged copy of the
tensor (rows and columns cut inside a block) takes the edge-tile code path over the same values.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_11170_amd as gws
from paper_2505_11170_amd import synth
from gpu_util import DEV, ensure_built

pytestmark = pytest.mark.gpu

# block maxima as BF16 bit patterns: 1.0, ~0.0201 (odd mantissa), 1.75, 0.0622 (mantissa all ones), 2^-99, 2^40.
# (2^-99 and not the 2^-100 that bounds the supported domain: in the ragged copy an edge block can lose its planted
# maximum, and the largest remaining pattern must still lie in the domain.)
MAXIMA = [0x3F80, 0x3CA5, 0x3FE0, 0x3D7F, 0x0E00, 0x5380]
BITWIDTHS = [60.0, 6.0, 2.0, 1.0]
NBC = 8                                   # blocks per block row: 256 columns = one workgroup tile


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def build_tensor():
    """Returns (w uint16 [rows, 256], b_t float32 [rows/32, 8]) as described in the module docstring."""
    rng = np.random.default_rng(65280)
    blocks, bts = [], []
    for a16 in MAXIMA:
        mags = np.arange(0, a16 + 1, dtype=np.uint16)                       # every magnitude pattern up to the maximum
        pats = np.concatenate([mags, mags | 0x8000])                        # ... with both signs
        for bt in BITWIDTHS:
            p = rng.permutation(pats)
            n_blk = -(-len(p) // 1023)
            p = np.concatenate([p, p[: n_blk * 1023 - len(p)]])             # fill the last slice with repeats
            for k in range(n_blk):
                blk = np.insert(p[k * 1023:(k + 1) * 1023], int(rng.integers(0, 1024)), a16)   # plant the maximum
                blocks.append(blk.reshape(32, 32))
                bts.append(bt)
    while len(blocks) % NBC:                                                # complete the last block row
        blocks.append(blocks[-1])
        bts.append(bts[-1])
    nbr = len(blocks) // NBC
    w = np.block([[blocks[i * NBC + j] for j in range(NBC)] for i in range(nbr)]).astype(np.uint16)
    return np.ascontiguousarray(w), np.asarray(bts, dtype=np.float32).reshape(nbr, NBC)


@pytest.fixture(scope="module")
def sweep():
    w, bt = build_tensor()
    seen = np.unique(w)
    assert len(seen) == 2 * (max(MAXIMA) + 1)                               # all patterns up to the largest maximum, +-
    return w, bt


@pytest.mark.parametrize("fmt", [gws.FMT_FP8_E4M3, gws.FMT_FP6_E3M2], ids=["fp8_e4m3", "fp6_e3m2"])
@pytest.mark.parametrize("ragged", [False, True], ids=["full_tiles", "edge_tiles"])
def test_every_bf16_pattern_through_the_cast(sweep, fmt, ragged):
    w_all, bt_all = sweep
    seed, step = oracle.derive_seed(65, 280), 9
    if ragged:                                                              # cut inside the last block row and column
        rows, cols = w_all.shape[0] - 13, w_all.shape[1] - 21
    else:
        rows, cols = w_all.shape
    ld = w_all.shape[1]
    w_np = np.ascontiguousarray(w_all[:rows])
    nbr, nbc = synth.n_blocks(rows, cols)
    bt_np = np.ascontiguousarray(bt_all[:nbr, :nbc])
    w = synth.from_bits(w_np, DEV)
    bt = torch.from_numpy(bt_np).to(DEV)
    w_hat = w.clone()
    scale = torch.full((nbr, nbc), float("nan"), device=DEV)
    d = gws.TensorDesc(rows=rows, cols=cols, ld=ld, seed=seed, w=w, w_hat=w_hat, bt=bt, scale=scale)
    gws.gws_sample_fwd([d], fmt, step)
    ldc = oracle.mx_row_bytes(cols, fmt) + 8                               # padded rows: FP8 a multiple of 8, FP6 of 2
    ldc = (ldc + 7) // 8 * 8 if fmt == gws.FMT_FP8_E4M3 else (ldc + 1) // 2 * 2
    codes = torch.full((rows, ldc), 0xAA, dtype=torch.uint8, device=DEV)
    xscale = torch.zeros(nbr, nbc, dtype=torch.uint8, device=DEV)
    scale_mx = torch.full((nbr, nbc), float("nan"), device=DEV)
    gws.gws_sample_fwd_mx([gws.TensorDesc(rows=rows, cols=cols, ld=ld, seed=seed, w=w, bt=bt, scale=scale_mx)],
                          [gws.MxOut(codes, xscale, ldc)], fmt, step)
    torch.cuda.synchronize()

    ref_q, ref_s = oracle.sample_fwd(w_np, bt_np, fmt, seed, step, cols=cols)
    amax = np.array([[(w_np[i * 32:i * 32 + 32, j * 32:min(cols, j * 32 + 32)] & 0x7FFF).max() for j in range(nbc)] for i in range(nbr)])
    assert amax.min() >= 0x0D80                                             # every block inside the supported domain
    got = synth.bits(w_hat)
    bad = np.argwhere(got != ref_q)
    assert len(bad) == 0, [(int(i), int(j), hex(w_np[i, j]), float(bt_np[i // 32, j // 32]), hex(got[i, j]), hex(ref_q[i, j]))
                           for i, j in bad[:8]]
    assert (scale.cpu().numpy().view(np.uint32) == ref_s.view(np.uint32)).all()
    ref_c, ref_x, ref_s2 = oracle.sample_fwd_mx(w_np, bt_np, fmt, seed, step, cols=cols, ldc=ldc)
    got_c = codes.cpu().numpy()
    badc = np.argwhere(got_c != ref_c)
    assert len(badc) == 0, [(int(i), int(j), hex(got_c[i, j]), hex(ref_c[i, j])) for i, j in badc[:8]]
    assert (xscale.cpu().numpy() == ref_x).all()
    assert (scale_mx.cpu().numpy().view(np.uint32) == ref_s2.view(np.uint32)).all()

    # the sweep did reach what it is for: saturated outputs (b_t = 2), target subnormals and zeros from underflow
    wv = (w_np.astype(np.uint32) << 16).view(np.float32).astype(np.float64)[:, :cols]
    qv = (ref_q.astype(np.uint32) << 16).view(np.float32).astype(np.float64)[:, :cols]
    assert ((qv == 0) & (wv != 0)).sum() > 1000                            # underflow to zero
    emax_v = 448.0 if fmt == gws.FMT_FP8_E4M3 else 28.0
    top = np.repeat(np.repeat(np.exp2(ref_x.astype(np.float64) - 127.0), 32, axis=0), 32, axis=1)[:rows, :cols] * emax_v
    assert (np.abs(qv) == top).sum() > 10                                  # saturation at the largest code
