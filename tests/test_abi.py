"""Host-side checks of the C ABI: the library loads, exports every symbol that
include/gws.h declares, validates arguments before any launch, and derives seeds
like the oracle.  No GPU work is issued here."""
import ctypes
import os
import re

import pytest

import oracle
from paper_2505_11170_amd import binding
from paper_2505_11170_amd.binding import _CBitwidth, _CMxOut, _CTensor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        from paper_2505_11170_amd.build import build_library
        build_library()
    return binding.load_library()


def declared_symbols(header="gws.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gws_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"gws_sample_fwd", "gws_sample_bwd", "gws_linear_fwd"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.EXPORTS)
    assert lib.gws_version() >= 1
    # the method's header lists no measurement aid; those live in their own header
    bench = declared_symbols("gws_bench.h")
    assert set(bench) == set(binding.BENCH_EXPORTS) and not set(bench) & set(names)
    for n in bench:
        assert hasattr(lib, n), n


def test_derive_seed_matches_oracle(lib):
    for u, t in [(0, 0), (0, 1), (1, 0), (0xDEADBEEF12345678, 0x1_00000002), (2 ** 64 - 1, 2 ** 64 - 1)]:
        assert binding.gws_derive_seed(u, t) == oracle.derive_seed(u, t)


def _t(**kw):
    c = _CTensor()
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def test_argument_validation_launches_nothing(lib):
    OK, NULL, SHAPE, ALIGN, FORMAT, LAUNCH, ALIAS = range(7)
    fake = 0x10000  # never dereferenced: every case below fails validation first
    base = dict(w=fake, w_hat=fake + 0x100000, bt=fake, scale=fake, g=fake, dw=None, dbt=fake,
                rows=64, cols=64, ld=64, row0=0, col0=0, seed=1)

    def fwd(fmt=1, **over):
        arr = (_CTensor * 1)(_t(**{**base, **over}))
        return lib.gws_sample_fwd(arr, 1, fmt, 0, None)

    def bwd(**over):
        arr = (_CTensor * 1)(_t(**{**base, **over}))
        return lib.gws_sample_bwd(arr, 1, 0, None)

    assert lib.gws_sample_fwd(None, 0, 1, 0, None) == OK          # empty list
    assert lib.gws_sample_fwd(None, 1, 1, 0, None) == NULL
    assert lib.gws_sample_fwd(None, -1, 1, 0, None) == SHAPE
    assert fwd(rows=0) == OK and fwd(cols=0) == OK and bwd(rows=0) == OK   # empty tensors are skipped
    assert fwd(w=None) == NULL and fwd(w_hat=None) == NULL and fwd(bt=None) == NULL and fwd(scale=None) == NULL
    assert fwd(fmt=3) == FORMAT and fwd(fmt=-1) == FORMAT
    assert fwd(ld=60) == SHAPE and fwd(ld=56) == SHAPE and fwd(rows=-1) == SHAPE and fwd(cols=2 ** 31) == SHAPE
    assert fwd(row0=16) == SHAPE and fwd(col0=8) == SHAPE and fwd(row0=-32) == SHAPE
    assert fwd(w=fake + 2) == ALIGN and fwd(w_hat=fake + 0x100008) == ALIGN and fwd(bt=fake + 1) == ALIGN
    assert fwd(w_hat=fake) == ALIAS and fwd(w_hat=fake + 64) == ALIAS
    assert bwd(g=None) == NULL and bwd(dbt=None) == NULL and bwd(scale=None) == NULL
    assert bwd(g=fake + 4) == ALIGN and bwd(dw=fake + 32) == ALIAS
    assert bwd(ld=63) == SHAPE
    assert lib.gws_noise_packed(None, 4, 4, 0, 0, 0, 0, None) == NULL
    assert lib.gws_noise_packed(fake, 4, 4, 0, 4, 0, 0, None) == SHAPE
    assert lib.gws_noise_packed(None, 0, 4, 0, 0, 0, 0, None) == OK
    # linear: shape rules
    wdesc = (_CTensor * 1)(_t(**base))
    assert lib.gws_linear_fwd(fake, 8, 32, 32, wdesc, 0, 1, 0, fake, 64, None) == SHAPE      # K mismatch
    assert lib.gws_linear_fwd(fake, 8, 64, 64, wdesc, 0, 9, 0, fake, 64, None) == FORMAT
    assert lib.gws_linear_fwd_mode(fake, 8, 64, 64, wdesc, 0, 1, 0, fake, 64, 4, None) == FORMAT    # no such mode
    assert lib.gws_linear_fwd_mode(fake, 8, 64, 64, wdesc, 0, 1, 0, fake, 64, -1, None) == FORMAT
    assert lib.gws_linear_fwd_mode(fake, 8, 64, 64, wdesc, 0, 1, 0, fake, 64, 1, None) == FORMAT    # a retired mode value
    assert lib.gws_linear_fwd_mode(fake, 0, 64, 64, wdesc, 0, 1, 0, fake, 64, 3, None) == OK        # empty
    # linear with w_hat staged in a workspace: the workspace is checked like any buffer
    need = lib.gws_linear_fwd_workspace_bytes(wdesc)
    assert need == 64 * 64 * 2 + 4 * 4 and lib.gws_linear_fwd_workspace_bytes(None) == 0
    ws = fake + 0x900000
    lin = (fake + 0x300000, 8, 64, 64, wdesc, 0, 1, 0, fake + 0x500000, 64)
    assert lib.gws_linear_fwd_ws(*lin, None, need, None) == NULL
    assert lib.gws_linear_fwd_ws(*lin, ws + 16, need, None) == ALIGN
    assert lib.gws_linear_fwd_ws(*lin, ws, need - 1, None) == SHAPE
    assert lib.gws_linear_fwd_ws(*lin, fake, need, None) == ALIAS                                  # workspace on w
    assert lib.gws_linear_fwd_ws(*lin, fake + 0x500000, need, None) == ALIAS                       # workspace on y
    assert lib.gws_linear_fwd_ws(fake, 0, 64, 64, wdesc, 0, 1, 0, fake, 64, None, 0, None) == OK   # empty
    # the allocation-free form: same argument rules; a weight beyond the library's staging buffer is refused
    TOO_LARGE = 7
    assert lib.gws_linear_fwd_static(None, 8, 64, 64, wdesc, 0, 1, 0, fake + 0x500000, 64, None) == NULL
    assert lib.gws_linear_fwd_static(fake + 0x300000, 8, 32, 32, wdesc, 0, 1, 0, fake + 0x500000, 64, None) == SHAPE
    assert lib.gws_linear_fwd_static(fake, 0, 64, 64, wdesc, 0, 1, 0, fake, 64, None) == OK        # empty
    big = (_CTensor * 1)(_t(**{**base, "rows": 4096, "cols": 4096 + 32, "ld": 4096 + 32}))         # 33 MiB of w_hat
    assert lib.gws_linear_fwd_workspace_bytes(big) > 32 << 20
    assert lib.gws_linear_fwd_static(fake + 0x300000, 8, 4096, 4096, big, 0, 1, 0, fake + 0x500000, 4128, None) == TOO_LARGE
    assert lib.gws_gemm_bf16(fake, 8, 48, 48, fake, 64, 64, 0, fake, 64, None) == SHAPE      # K % 32
    assert lib.gws_gemm_bf16(None, 8, 64, 64, fake, 64, 64, 0, fake, 64, None) == NULL
    assert lib.gws_gemm_bf16(fake, 0, 64, 64, fake, 64, 64, 0, fake, 64, None) == OK         # empty
    # GEMM with the next weight's sampling: the next weight is checked like gws_sample_fwd's, and may not
    # overlap the GEMM's operands
    nxt = (_CTensor * 1)(_t(**base))
    gemm = (fake, 256, 64, 64, fake + 0x400000, 256, 256, 0, fake + 0x800000, 256)
    assert lib.gws_gemm_bf16_sample_next(*gemm, nxt, 9, 0, None) == FORMAT
    assert lib.gws_gemm_bf16_sample_next(*gemm, (_CTensor * 1)(_t(**{**base, "bt": None})), 1, 0, None) == NULL
    assert lib.gws_gemm_bf16_sample_next(*gemm, (_CTensor * 1)(_t(**{**base, "w_hat": fake + 0x400000})), 1, 0, None) == ALIAS
    assert lib.gws_gemm_bf16_sample_next(*gemm, (_CTensor * 1)(_t(**{**base, "w_hat": fake + 0x800040})), 1, 0, None) == ALIAS
    assert lib.gws_gemm_bf16_sample_next(fake, 256, 48, 48, fake + 0x400000, 256, 256, 0, fake + 0x800000, 256, nxt, 1, 0, None) == SHAPE
    assert lib.gws_gemm_bf16_sample_next(None, 256, 64, 64, fake + 0x400000, 256, 256, 0, fake + 0x800000, 256, nxt, 1, 0, None) == NULL
    for s in range(8):
        assert lib.gws_status_string(s)


def test_bitwidth_and_mx_entry_points_validate_before_any_launch(lib):
    OK, NULL, SHAPE, ALIGN, FORMAT, LAUNCH, ALIAS = range(7)
    fake = 0x10000  # never dereferenced: every case below fails validation first
    base = dict(w=fake, w_hat=fake + 0x100000, bt=fake, scale=fake, g=fake, dw=None, dbt=fake,
                rows=64, cols=64, ld=64, row0=0, col0=0, seed=1)
    bw = (_CBitwidth * 1)()
    bw[0].b_init, bw[0].b_target, bw[0].lam, bw[0].layer_blocks = 6.0, 4.0, 0.0, 0

    def arr(**over):
        return (_CTensor * 1)(_t(**{**base, **over}))

    assert lib.gws_sample_fwd_bi(arr(), 1, None, 1, 0, None) == NULL           # no bitwidth settings
    assert lib.gws_sample_fwd_bi(None, 0, None, 1, 0, None) == OK              # empty list
    assert lib.gws_sample_fwd_bi(arr(), 1, bw, 7, 0, None) == FORMAT
    assert lib.gws_sample_fwd_bi(arr(bt=None), 1, bw, 1, 0, None) == NULL
    assert lib.gws_sample_bwd_bi(arr(bt=None), 1, bw, 0, None) == NULL         # backward needs b_i here
    assert lib.gws_sample_bwd_bi(arr(bt=fake + 2), 1, bw, 0, None) == ALIGN
    bw[0].layer_blocks = -1
    assert lib.gws_sample_bwd_bi(arr(), 1, bw, 0, None) == SHAPE
    assert lib.gws_sample_bwd_bi(arr(rows=0), 1, bw, 0, None) == SHAPE         # checked for every tensor, empty or not

    def mx(fmt=1, codes=fake + 0x200000, xscale=fake, ldc=64, **over):
        o = (_CMxOut * 1)()
        o[0].codes, o[0].xscale, o[0].ldc = codes, xscale, ldc
        return lib.gws_sample_fwd_mx(arr(**over), o, 1, fmt, 0, None)

    assert mx(fmt=0) == FORMAT and mx(fmt=3) == FORMAT                         # MX exists for FP8 and FP6 only
    assert mx(codes=None) == NULL and mx(xscale=None) == NULL and mx(w=None) == NULL
    assert mx(w_hat=None, rows=0) == OK                                        # w_hat is not used; empty tensors are skipped
    assert mx(ldc=56) == SHAPE and mx(ldc=68) == SHAPE                         # FP8: >= cols, multiple of 8
    assert mx(fmt=2, ldc=46) == SHAPE and mx(fmt=2, ldc=49) == SHAPE           # FP6: >= 48 bytes, even
    assert mx(codes=fake + 0x200004) == ALIGN and mx(fmt=2, ldc=48, codes=fake + 0x200001) == ALIGN
    assert mx(codes=fake + 128) == ALIAS                                       # codes inside w
    assert lib.gws_sample_fwd_mx(arr(), None, 1, 1, 0, None) == NULL


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libgws.so"))
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        binding.load_library()
