"""GaussWS CPU oracle: TEST INFRASTRUCTURE ONLY.

ctypes front end of ``gws_oracle.c`` (plain C, fp64 reductions, integer-emulated
BF16 arithmetic).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product package
never does, and this package never imports the product.

BF16 tensors are exchanged as ``numpy.uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gws_oracle.c")
_LIB = os.path.join(_HERE, "libgws_oracle.so")

FMT_BF16, FMT_FP8_E4M3, FMT_FP6_E3M2 = 0, 1, 2
BASIS_BITS, BASIS_UNIFORM, BASIS_BOX_MULLER = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (host only, no HIP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def configure(L: ctypes.CDLL) -> ctypes.CDLL:
    """Declare the argument types of every entry point on a loaded oracle library."""
    u32p = ctypes.POINTER(ctypes.c_uint32)
    vp, i64, u64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int
    L.gwso_set_threads.argtypes = [ci]
    L.gwso_set_threads.restype = ci
    L.gwso_philox4x32.argtypes = [u32p, u32p, ci, u32p]
    L.gwso_philox4x32.restype = None
    L.gwso_derive_seed.argtypes = [u64, u64]
    L.gwso_derive_seed.restype = u64
    L.gwso_nibbles_to_code.argtypes = [ctypes.c_uint] * 4
    L.gwso_nibbles_to_code.restype = ci
    L.gwso_code_to_r.argtypes = [ci]
    L.gwso_code_to_r.restype = ci
    L.gwso_element_nibble.argtypes = [ci]
    L.gwso_element_nibble.restype = ci
    L.gwso_noise.argtypes = [i64, i64, i64, i64, u64, u64, vp, vp]
    L.gwso_noise.restype = None
    L.gwso_bf16_rne.argtypes = [ctypes.c_float]
    L.gwso_bf16_rne.restype = ctypes.c_uint16
    L.gwso_bf16_add.argtypes = [ctypes.c_uint16, ctypes.c_uint16]
    L.gwso_bf16_add.restype = ctypes.c_uint16
    L.gwso_exp2.argtypes = [ctypes.c_float]
    L.gwso_exp2.restype = ctypes.c_float
    L.gwso_cast.argtypes = [ctypes.c_uint16, ci, ci]
    L.gwso_cast.restype = ctypes.c_uint16
    L.gwso_bf16_add_n.argtypes = [vp, vp, vp, i64]
    L.gwso_bf16_add_n.restype = None
    L.gwso_cast_n.argtypes = [vp, ci, ci, vp, i64]
    L.gwso_cast_n.restype = None
    L.gwso_exp2_n.argtypes = [vp, vp, i64]
    L.gwso_exp2_n.restype = None
    L.gwso_sample_fwd.argtypes = [vp, i64, i64, i64, i64, i64, vp, ci, u64, u64, vp, vp]
    L.gwso_sample_fwd.restype = ci
    L.gwso_sample_bwd.argtypes = [vp, i64, i64, i64, i64, i64, vp, u64, u64, vp, vp, vp]
    L.gwso_sample_bwd.restype = ci
    L.gwso_sample_fwd_basis.argtypes = [vp, i64, i64, i64, i64, i64, vp, ci, ci, u64, u64, vp, vp]
    L.gwso_sample_fwd_basis.restype = ci
    L.gwso_sample_bwd_basis.argtypes = [vp, i64, i64, i64, i64, i64, vp, ci, u64, u64, vp, vp, vp]
    L.gwso_sample_bwd_basis.restype = ci
    L.gwso_uniform_bf16.argtypes = [ctypes.c_uint]
    L.gwso_uniform_bf16.restype = ctypes.c_uint16
    L.gwso_bf16_mul.argtypes = [ctypes.c_uint16, ctypes.c_uint16]
    L.gwso_bf16_mul.restype = ctypes.c_uint16
    L.gwso_box_muller.argtypes = [ctypes.c_uint32, ctypes.POINTER(ctypes.c_float)]
    L.gwso_box_muller.restype = None
    L.gwso_box_muller_n.argtypes = [vp, vp, i64]
    L.gwso_box_muller_n.restype = None
    L.gwso_noise_basis.argtypes = [i64, i64, i64, i64, u64, u64, ci, vp]
    L.gwso_noise_basis.restype = None
    L.gwso_linear_fwd.argtypes = [vp, i64, i64, i64, vp, i64, i64, ci, vp, i64, vp, vp, vp]
    L.gwso_linear_fwd.restype = ci
    L.gwso_mx_code_value.argtypes = [ci, ci]
    L.gwso_mx_code_value.restype = ctypes.c_double
    L.gwso_mx_encode.argtypes = [ctypes.c_uint16, ci, ci]
    L.gwso_mx_encode.restype = ci
    L.gwso_sample_fwd_mx.argtypes = [vp, i64, i64, i64, i64, i64, vp, ci, u64, u64, vp, i64, vp, vp]
    L.gwso_sample_fwd_mx.restype = ci
    L.gwso_bitwidth.argtypes = [vp, i64, ctypes.c_float, ctypes.c_float, vp]
    L.gwso_bitwidth.restype = None
    L.gwso_bitwidth_grad.argtypes = [vp, vp, i64, ctypes.c_float, ctypes.c_float, ctypes.c_double, i64, vp]
    L.gwso_bitwidth_grad.restype = None
    return L


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = configure(ctypes.CDLL(_LIB))
    return _lib


def set_threads(n: int) -> int:
    return lib().gwso_set_threads(int(n))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def philox4x32(ctr, key, rounds: int = 10):
    c = (ctypes.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (ctypes.c_uint32 * 4)()
    lib().gwso_philox4x32(c, k, rounds, o)
    return [int(v) for v in o]


def derive_seed(user_seed: int, tensor_id: int) -> int:
    return int(lib().gwso_derive_seed(user_seed & (2**64 - 1), tensor_id & (2**64 - 1)))


def nibbles_to_code(n0, n1, n2, n3) -> int:
    return int(lib().gwso_nibbles_to_code(n0, n1, n2, n3))


def code_to_r(code: int) -> int:
    return int(lib().gwso_code_to_r(code))


def element_nibble(k: int) -> int:
    return int(lib().gwso_element_nibble(k))


def noise(rows: int, cols: int, seed: int, step: int, row0: int = 0, col0: int = 0):
    """Returns (R int8 [rows, cols], packed uint32 [rows, ceil(cols/8)])."""
    assert col0 % 8 == 0
    r = np.empty((rows, cols), dtype=np.int8)
    packed = np.empty((rows, (cols + 7) // 8), dtype=np.uint32)
    lib().gwso_noise(rows, cols, row0, col0, seed, step, _ptr(r), _ptr(packed))
    return r, packed


def bf16_rne(f: float) -> int:
    return int(lib().gwso_bf16_rne(f))


def bf16_add(a: int, b: int) -> int:
    return int(lib().gwso_bf16_add(a, b))


def exp2(t: float) -> float:
    return float(lib().gwso_exp2(t))


def cast(v16: int, Ea: int, fmt: int) -> int:
    return int(lib().gwso_cast(v16, Ea, fmt))


def bf16_add_n(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.uint16)
    b = np.ascontiguousarray(b, dtype=np.uint16)
    assert a.shape == b.shape
    out = np.empty_like(a)
    lib().gwso_bf16_add_n(_ptr(a), _ptr(b), _ptr(out), a.size)
    return out


def cast_n(v: np.ndarray, Ea: int, fmt: int) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.uint16)
    out = np.empty_like(v)
    lib().gwso_cast_n(_ptr(v), Ea, fmt, _ptr(out), v.size)
    return out


def exp2_n(t: np.ndarray) -> np.ndarray:
    t = np.ascontiguousarray(t, dtype=np.float32)
    out = np.empty_like(t)
    lib().gwso_exp2_n(_ptr(t), _ptr(out), t.size)
    return out


def n_blocks(rows: int, cols: int):
    return (rows + 31) // 32, (cols + 31) // 32


def uniform_bf16(byte: int) -> int:
    """BF16 bits of the uniform basis value (2 * byte - 255) / 512."""
    return int(lib().gwso_uniform_bf16(int(byte)))


def bf16_mul(a: int, b: int) -> int:
    return int(lib().gwso_bf16_mul(a, b))


def box_muller(words: np.ndarray) -> np.ndarray:
    """uint32 words -> float32 [n, 2]: the two standard normals each word gives (fp32, the oracle's defined sequence)."""
    words = np.ascontiguousarray(words, dtype=np.uint32)
    z = np.empty((words.size, 2), dtype=np.float32)
    lib().gwso_box_muller_n(_ptr(words), _ptr(z), words.size)
    return z


def noise_basis(rows: int, cols: int, seed: int, step: int, basis: int, row0: int = 0, col0: int = 0) -> np.ndarray:
    """R of every element under a basis, float32 [rows, cols]."""
    r = np.empty((rows, cols), dtype=np.float32)
    lib().gwso_noise_basis(rows, cols, row0, col0, seed, step, basis, _ptr(r))
    return r


def sample_fwd(w: np.ndarray, bt: np.ndarray, fmt: int, seed: int, step: int, cols: int | None = None,
               row0: int = 0, col0: int = 0, basis: int = BASIS_BITS):
    """w: uint16 [rows, ld] (BF16 bits), bt: float32 [nbr, nbc].
    `cols` defaults to w.shape[1] (= ld).  Returns (w_hat uint16 like w, scale float32).
    `basis` other than BASIS_BITS draws R from one of the comparison bases."""
    assert w.dtype == np.uint16 and w.ndim == 2 and w.flags.c_contiguous
    rows, ld = w.shape
    cols = ld if cols is None else cols
    nbr, nbc = n_blocks(rows, cols)
    bt = np.ascontiguousarray(bt, dtype=np.float32).reshape(nbr, nbc)
    w_hat = w.copy()  # padding columns (>= cols) keep the input bytes
    scale = np.empty((nbr, nbc), dtype=np.float32)
    if basis == BASIS_BITS:
        rc = lib().gwso_sample_fwd(_ptr(w), rows, cols, ld, row0, col0, _ptr(bt), fmt, seed, step, _ptr(w_hat), _ptr(scale))
    else:
        rc = lib().gwso_sample_fwd_basis(_ptr(w), rows, cols, ld, row0, col0, _ptr(bt), fmt, basis, seed, step,
                                         _ptr(w_hat), _ptr(scale))
    if rc:
        raise RuntimeError(f"gwso_sample_fwd status {rc}")
    return w_hat, scale


def sample_bwd(g: np.ndarray, scale: np.ndarray, seed: int, step: int, cols: int | None = None,
               row0: int = 0, col0: int = 0, basis: int = BASIS_BITS):
    """g: uint16 [rows, ld].  Returns (dw uint16, dbt float64 [nbr,nbc], abs_sum float64)."""
    assert g.dtype == np.uint16 and g.ndim == 2 and g.flags.c_contiguous
    rows, ld = g.shape
    cols = ld if cols is None else cols
    nbr, nbc = n_blocks(rows, cols)
    scale = np.ascontiguousarray(scale, dtype=np.float32).reshape(nbr, nbc)
    dw = np.zeros_like(g)
    dbt = np.empty((nbr, nbc), dtype=np.float64)
    asum = np.empty((nbr, nbc), dtype=np.float64)
    if basis == BASIS_BITS:
        rc = lib().gwso_sample_bwd(_ptr(g), rows, cols, ld, row0, col0, _ptr(scale), seed, step, _ptr(dw), _ptr(dbt), _ptr(asum))
    else:
        rc = lib().gwso_sample_bwd_basis(_ptr(g), rows, cols, ld, row0, col0, _ptr(scale), basis, seed, step,
                                         _ptr(dw), _ptr(dbt), _ptr(asum))
    if rc:
        raise RuntimeError(f"gwso_sample_bwd status {rc}")
    return dw, dbt, asum


def mx_code_value(code: int, fmt: int) -> float:
    return float(lib().gwso_mx_code_value(code, fmt))


def mx_encode(q16: int, Ea: int, fmt: int) -> int:
    return int(lib().gwso_mx_encode(q16, Ea, fmt))


def mx_row_bytes(cols: int, fmt: int) -> int:
    return cols if fmt == FMT_FP8_E4M3 else (cols * 6 + 7) // 8


def sample_fwd_mx(w: np.ndarray, bt: np.ndarray, fmt: int, seed: int, step: int, cols: int | None = None,
                  row0: int = 0, col0: int = 0, ldc: int | None = None):
    """Forward pass with MX output.  Returns (codes uint8 [rows, ldc], xscale uint8 [nbr, nbc], scale float32).
    Bytes of `codes` past a row's data keep the fill value 0xAA."""
    assert w.dtype == np.uint16 and w.ndim == 2 and w.flags.c_contiguous
    rows, ld = w.shape
    cols = ld if cols is None else cols
    nbr, nbc = n_blocks(rows, cols)
    bt = np.ascontiguousarray(bt, dtype=np.float32).reshape(nbr, nbc)
    ldc = mx_row_bytes(cols, fmt) if ldc is None else ldc
    codes = np.full((rows, ldc), 0xAA, dtype=np.uint8)
    xscale = np.zeros((nbr, nbc), dtype=np.uint8)
    scale = np.empty((nbr, nbc), dtype=np.float32)
    rc = lib().gwso_sample_fwd_mx(_ptr(w), rows, cols, ld, row0, col0, _ptr(bt), fmt, seed, step, _ptr(codes), ldc,
                                  _ptr(xscale), _ptr(scale))
    if rc:
        raise RuntimeError(f"gwso_sample_fwd_mx status {rc}")
    return codes, xscale, scale


def bitwidth(bi: np.ndarray, b_init: float, b_target: float) -> np.ndarray:
    """Eq. 11 in fp32: b_t = b_target + b_i * (b_init - b_target)."""
    bi = np.ascontiguousarray(bi, dtype=np.float32)
    bt = np.empty_like(bi)
    lib().gwso_bitwidth(_ptr(bi), bi.size, b_init, b_target, _ptr(bt))
    return bt


def bitwidth_grad(bi: np.ndarray, dbt: np.ndarray, b_init: float, b_target: float, lam: float, m: int) -> np.ndarray:
    """dL'/db_i of Eq. 12 (fp64) for blocks of a layer of m blocks, from dL/db_t."""
    bi = np.ascontiguousarray(bi, dtype=np.float32)
    dbt = np.ascontiguousarray(dbt, dtype=np.float64)
    assert bi.shape == dbt.shape
    dbi = np.empty_like(dbt)
    lib().gwso_bitwidth_grad(_ptr(bi), _ptr(dbt), bi.size, b_init, b_target, lam, m, _ptr(dbi))
    return dbi


def linear_fwd(x: np.ndarray, q: np.ndarray, w_is_nk: bool = False, rows_sel=None):
    """x: uint16 [M, K]; q: uint16 [K, N] (or [N, K] if w_is_nk).
    Returns (y64 [R, N], yabs [R, N], y16 uint16 [R, N]) for the selected rows."""
    assert x.dtype == np.uint16 and q.dtype == np.uint16
    M, K = x.shape
    N = q.shape[0] if w_is_nk else q.shape[1]
    assert (q.shape[1] if w_is_nk else q.shape[0]) == K
    sel = None if rows_sel is None else np.ascontiguousarray(rows_sel, dtype=np.int64)
    R = M if sel is None else len(sel)
    y64 = np.empty((R, N), dtype=np.float64)
    yabs = np.empty((R, N), dtype=np.float64)
    y16 = np.empty((R, N), dtype=np.uint16)
    rc = lib().gwso_linear_fwd(_ptr(x), M, K, x.shape[1], _ptr(q), N, q.shape[1], int(w_is_nk),
                               _ptr(sel), R, _ptr(y64), _ptr(yabs), _ptr(y16))
    if rc:
        raise RuntimeError(f"gwso_linear_fwd status {rc}")
    return y64, yabs, y16
