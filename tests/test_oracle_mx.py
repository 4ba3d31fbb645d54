"""Pins of the oracle's microscaling (MX) output: element codes and E8M0 block scales.

What fixes the encodings, other than the oracle itself: torch's float8_e4m3fn byte patterns, the
figures the OCP Microscaling Formats specification (v1.0, element-format tables) prints for
FP6 E3M2 and FP8 E4M3, numpy's bit unpacking for the 6-bit layout, numpy's frexp for the shared
exponent, and the already pinned BF16-container output of the forward pass.  CPU only."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_11170_amd import synth
from test_oracle_sample import bf16_val, block_absmax, to_bits

E4M3, E3M2 = oracle.FMT_FP8_E4M3, oracle.FMT_FP6_E3M2


def test_e4m3_code_values_match_torch_float8():
    codes = np.arange(256, dtype=np.uint8)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    for c in range(256):
        if c & 0x7F == 0x7F:
            assert np.isnan(ref[c])          # the one NaN pattern per sign: never produced by the method
            continue
        assert oracle.mx_code_value(c, E4M3) == ref[c], c


def test_e3m2_code_values_match_the_specification_figures():
    val = [oracle.mx_code_value(c, E3M2) for c in range(64)]
    # printed in the specification for E3M2 (exponent bias 3): max normal 28, min normal 0.25,
    # max subnormal 0.1875, min subnormal 0.0625; 1.0 is S.011.00
    assert val[0b011111] == 28.0 and val[0b000100] == 0.25 and val[0b000011] == 0.1875 and val[0b000001] == 0.0625
    assert val[0b001100] == 1.0 and val[0] == 0.0
    mags = np.array(val[:32])
    assert (np.diff(mags) > 0).all()                                  # code order is value order
    d = np.diff(mags)
    assert (d[:8] == 0.0625).all()                                    # subnormals and the first binade share a spacing
    for E in range(1, 8):                                             # four equal steps per binade, doubling
        steps = d[4 * E:4 * E + 4]                                   # within binade E and up to the next one
        assert len(steps) == (4 if E < 7 else 3) and (steps == 2.0 ** (E - 3 - 2)).all()
    assert val[32:] == [-v for v in val[:32]] and np.signbit(val[32])  # sign is the top bit; -0 exists


@pytest.mark.parametrize("fmt", [E4M3, E3M2])
def test_encode_inverts_the_code_values_at_any_block_scale(fmt):
    n = 256 if fmt == E4M3 else 64
    emax = 8 if fmt == E4M3 else 4
    for Ea in (-20, -6, 0, 3):
        X = 2.0 ** (Ea + 1 - emax)
        for c in range(n):
            if fmt == E4M3 and c & 0x7F == 0x7F:
                continue
            q16 = int(to_bits(np.array([oracle.mx_code_value(c, fmt) * X]))[0])
            if c == n // 2:
                q16 = 0x8000                 # -0.0
            assert oracle.mx_encode(q16, Ea, fmt) == c, (c, Ea)
    # a BF16 value that is not a member of X * format has no code
    assert oracle.mx_encode(int(to_bits(np.array([1.0 + 2.0 ** -7]))[0]), 0, fmt) == 0xFF


def test_e4m3_codes_of_cast_outputs_match_torch_on_every_bf16_input():
    v = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    finite = (v & 0x7F80) != 0x7F80
    for Ea in (-7, 0, 2):
        X = 2.0 ** (Ea + 1 - 8)
        q = oracle.cast_n(v, Ea, E4M3)
        y = torch.from_numpy((bf16_val(q) / X).astype(np.float32))
        ref = y.to(torch.float8_e4m3fn).view(torch.uint8).numpy()     # exact: q / X is a member of the format
        idx = np.nonzero(finite)[0][::17]
        got = np.array([oracle.mx_encode(int(q[i]), Ea, E4M3) for i in idx], dtype=np.uint8)
        assert np.array_equal(got, ref[idx])


def unpack_fp6(codes_row_bytes, cols):
    bits = np.unpackbits(codes_row_bytes, axis=1, bitorder="little")[:, :cols * 6]
    return (bits.reshape(bits.shape[0], cols, 6) * (1 << np.arange(6))).sum(axis=2)


@pytest.mark.parametrize("fmt", [E4M3, E3M2])
@pytest.mark.parametrize("shape", [(64, 96), (40, 50)])
def test_mx_output_decodes_to_the_bf16_container_output(fmt, shape):
    rows, cols = shape
    ld = (cols + 7) // 8 * 8
    t = synth.make_tensor(21, rows, cols, ld=ld)
    w, bt = synth.bits(t["w"]), t["bt"].numpy()
    seed, step = oracle.derive_seed(1, 21), 3
    q, s_ref = oracle.sample_fwd(w, bt, fmt, seed, step, cols=cols)
    codes, xscale, scale = oracle.sample_fwd_mx(w, bt, fmt, seed, step, cols=cols, ldc=oracle.mx_row_bytes(cols, fmt) + 3)
    assert np.array_equal(scale.view(np.uint32), s_ref.view(np.uint32))
    # shared exponent: floor(log2 max|w|) + 1 - emax, computed here with frexp
    emax = 8 if fmt == E4M3 else 4
    a = block_absmax(bf16_val(w)[:, :cols], rows, cols)
    Ea = np.frexp(a)[1] - 1
    assert np.array_equal(xscale.astype(np.int64) - 127, Ea + 1 - emax)
    # element codes, unpacked with numpy, decode to exactly the fake-quantised values
    nb = oracle.mx_row_bytes(cols, fmt)
    assert (codes[:, nb:] == 0xAA).all()                               # nothing written past a row's data
    c = codes[:, :cols].astype(np.int64) if fmt == E4M3 else unpack_fp6(codes[:, :nb], cols)
    val = np.array([oracle.mx_code_value(k, fmt) if not (fmt == E4M3 and k & 0x7F == 0x7F) else np.nan
                    for k in range(256 if fmt == E4M3 else 64)])
    X = np.repeat(np.repeat(2.0 ** (xscale.astype(np.float64) - 127), 32, axis=0), 32, axis=1)[:rows, :cols]
    dec = val[c] * X
    qv = bf16_val(q)[:, :cols]
    assert np.array_equal(dec, qv) and np.array_equal(np.signbit(dec), np.signbit(qv))
    if fmt == E3M2 and (cols * 6) % 8:
        used = (cols * 6) % 8                                          # unused bits of a row's last byte are 0
        assert (codes[:, nb - 1] >> used == 0).all()


def test_hand_block_scales():
    # max|w| = 1.0: X = 2^-7 for E4M3 (top binade [128, 256) * X = [1, 2)) and 2^-3 for E3M2
    w = to_bits(np.full((32, 32), 0.25))
    w[5, 7] = to_bits(np.array([-1.0]))[0]
    bt = np.full((1, 1), 6.0, dtype=np.float32)
    assert oracle.sample_fwd_mx(w, bt, E4M3, 1, 0)[1][0, 0] == 127 - 7
    assert oracle.sample_fwd_mx(w, bt, E3M2, 1, 0)[1][0, 0] == 127 - 3
    # all-zero block: X = 1, codes are signed zeros
    z = np.zeros((32, 32), dtype=np.uint16)
    z[0, 0] = 0x8000
    codes, xs, sc = oracle.sample_fwd_mx(z, bt, E4M3, 1, 0)
    assert xs[0, 0] == 127 and sc[0, 0] == 0.0 and set(np.unique(codes)) <= {0x00, 0x80}
