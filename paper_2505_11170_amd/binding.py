"""ctypes binding of ``libgws.so``: argument marshalling only.

Function names and argument order mirror ``include/gws.h``.  torch is used for
device memory and streams; every step of the method runs in the library's HIP
kernels.  There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("GWS_LIBRARY") or os.path.join(_HERE, "libgws.so")

FMT_BF16, FMT_FP8_E4M3, FMT_FP6_E3M2 = 0, 1, 2
LINEAR_AUTO, LINEAR_IN_OPERAND, LINEAR_TWO_KERNELS = 0, 2, 3
BASIS_BITS, BASIS_UNIFORM_BF16, BASIS_BOX_MULLER = 0, 1, 2

# include/gws.h (the method) and include/gws_bench.h (measurement aids)
EXPORTS = ("gws_sample_fwd", "gws_sample_bwd", "gws_sample_fwd_bi", "gws_sample_bwd_bi", "gws_sample_fwd_mx", "gws_linear_fwd", "gws_linear_fwd_mode",
           "gws_linear_fwd_ws", "gws_linear_fwd_workspace_bytes", "gws_linear_fwd_static", "gws_linear_bwd_w", "gws_linear_bwd_w_ws", "gws_linear_bwd_w_workspace_bytes", "gws_gemm_bf16", "gws_gemm_bf16_sample_next", "gws_gemm_bf16_sample_next_n", "gws_noise_packed",
           "gws_sample_fwd_basis", "gws_sample_bwd_basis", "gws_noise_basis",
           "gws_derive_seed", "gws_status_string", "gws_version")
BENCH_EXPORTS = ("gws_copy_tiles", "gws_block_absmax", "gws_sample_bwd_tuned", "gws_sample_fwd_tuned", "gws_gemm_bf16_ride_probe", "gws_ride_plan")


class GwsError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({status_string(status)})")
        self.status = status


class _CTensor(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("w_hat", ctypes.c_void_p), ("bt", ctypes.c_void_p),
                ("scale", ctypes.c_void_p), ("g", ctypes.c_void_p), ("dw", ctypes.c_void_p),
                ("dbt", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64), ("row0", ctypes.c_int64), ("col0", ctypes.c_int64),
                ("seed", ctypes.c_uint64)]


class _CBitwidth(ctypes.Structure):
    _fields_ = [("b_init", ctypes.c_float), ("b_target", ctypes.c_float), ("lam", ctypes.c_float),
                ("layer_blocks", ctypes.c_int64)]


class _CMxOut(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("xscale", ctypes.c_void_p), ("ldc", ctypes.c_int64)]


@dataclass
class MxOut:
    """Python-side mirror of ``gws_mx_out``: uint8 device tensors for element codes and E8M0 block scales."""
    codes: object
    xscale: object
    ldc: Optional[int] = None


@dataclass
class Bitwidth:
    """Python-side mirror of ``gws_bitwidth`` (paper Eq. 11 and Eq. 12), one per tensor."""
    b_init: float
    b_target: float
    lam: float = 0.0
    layer_blocks: int = 0


@dataclass
class TensorDesc:
    """Python-side mirror of ``gws_tensor``; tensor fields are torch device tensors or None."""
    rows: int
    cols: int
    seed: int
    w: Optional[object] = None
    w_hat: Optional[object] = None
    bt: Optional[object] = None
    scale: Optional[object] = None
    g: Optional[object] = None
    dw: Optional[object] = None
    dbt: Optional[object] = None
    ld: Optional[int] = None
    row0: int = 0
    col0: int = 0


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libgws.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2505_11170_amd.build` "
            "(hipcc, gfx950). There is no CPU or PyTorch fallback.")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i64, u64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int
    tp = ctypes.POINTER(_CTensor)
    L.gws_sample_fwd.argtypes = [tp, ci, ci, u64, vp]
    L.gws_sample_fwd.restype = ci
    L.gws_sample_bwd.argtypes = [tp, ci, u64, vp]
    L.gws_sample_bwd.restype = ci
    bp = ctypes.POINTER(_CBitwidth)
    L.gws_sample_fwd_bi.argtypes = [tp, ci, bp, ci, u64, vp]
    L.gws_sample_fwd_bi.restype = ci
    L.gws_sample_bwd_bi.argtypes = [tp, ci, bp, u64, vp]
    L.gws_sample_bwd_bi.restype = ci
    L.gws_sample_fwd_mx.argtypes = [tp, ctypes.POINTER(_CMxOut), ci, ci, u64, vp]
    L.gws_sample_fwd_mx.restype = ci
    L.gws_linear_fwd.argtypes = [vp, i64, i64, i64, tp, ci, ci, u64, vp, i64, vp]
    L.gws_linear_fwd.restype = ci
    L.gws_linear_fwd_mode.argtypes = [vp, i64, i64, i64, tp, ci, ci, u64, vp, i64, ci, vp]
    L.gws_linear_fwd_mode.restype = ci
    L.gws_linear_fwd_ws.argtypes = [vp, i64, i64, i64, tp, ci, ci, u64, vp, i64, vp, ctypes.c_size_t, vp]
    L.gws_linear_fwd_ws.restype = ci
    L.gws_linear_fwd_static.argtypes = [vp, i64, i64, i64, tp, ci, ci, u64, vp, i64, vp]
    L.gws_linear_fwd_static.restype = ci
    L.gws_linear_fwd_workspace_bytes.argtypes = [tp]
    L.gws_linear_fwd_workspace_bytes.restype = ctypes.c_size_t
    L.gws_gemm_bf16_sample_next.argtypes = [vp, i64, i64, i64, vp, i64, i64, ci, vp, i64, tp, ci, u64, vp]
    L.gws_gemm_bf16_sample_next.restype = ci
    L.gws_copy_tiles.argtypes = [tp, ci, vp]
    L.gws_copy_tiles.restype = ci
    L.gws_gemm_bf16_sample_next_n.argtypes = [vp, i64, i64, i64, vp, i64, i64, ci, vp, i64, tp, ci, ci, u64, vp]
    L.gws_gemm_bf16_sample_next_n.restype = ci
    L.gws_ride_plan.argtypes = [i64, i64, i64, tp, ci]
    L.gws_ride_plan.restype = ci
    L.gws_gemm_bf16_ride_probe.argtypes = [vp, i64, i64, i64, vp, i64, i64, ci, vp, i64, tp, ci, u64, ci, ci, vp]
    L.gws_gemm_bf16_ride_probe.restype = ci
    L.gws_sample_fwd_tuned.argtypes = [tp, ci, ci, u64, ci, ci, vp]
    L.gws_sample_fwd_tuned.restype = ci
    L.gws_sample_bwd_tuned.argtypes = [tp, ci, u64, ci, ci, vp]
    L.gws_sample_bwd_tuned.restype = ci
    L.gws_block_absmax.argtypes = [tp, ci, vp]
    L.gws_block_absmax.restype = ci
    L.gws_linear_bwd_w.argtypes = [vp, vp, i64, i64, i64, tp, ci, u64, vp]
    L.gws_linear_bwd_w.restype = ci
    L.gws_linear_bwd_w_workspace_bytes.argtypes = [tp, i64]
    L.gws_linear_bwd_w_workspace_bytes.restype = ctypes.c_size_t
    L.gws_linear_bwd_w_ws.argtypes = [vp, vp, i64, i64, i64, tp, ci, u64, vp, ctypes.c_size_t, vp]
    L.gws_linear_bwd_w_ws.restype = ci
    L.gws_gemm_bf16.argtypes = [vp, i64, i64, i64, vp, i64, i64, ci, vp, i64, vp]
    L.gws_gemm_bf16.restype = ci
    L.gws_sample_fwd_basis.argtypes = [tp, ci, ci, ci, u64, vp]
    L.gws_sample_fwd_basis.restype = ci
    L.gws_sample_bwd_basis.argtypes = [tp, ci, ci, u64, vp]
    L.gws_sample_bwd_basis.restype = ci
    L.gws_noise_basis.argtypes = [vp, i64, i64, i64, i64, u64, u64, ci, vp]
    L.gws_noise_basis.restype = ci
    L.gws_noise_packed.argtypes = [vp, i64, i64, i64, i64, u64, u64, vp]
    L.gws_noise_packed.restype = ci
    L.gws_derive_seed.argtypes = [u64, u64]
    L.gws_derive_seed.restype = u64
    L.gws_status_string.argtypes = [ci]
    L.gws_status_string.restype = ctypes.c_char_p
    L.gws_version.argtypes = []
    L.gws_version.restype = ci
    _lib = L
    return L


def status_string(status: int) -> str:
    try:
        return load_library().gws_status_string(int(status)).decode()
    except Exception:  # pragma: no cover
        return "?"


def _p(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


class PackedTensors:
    """A descriptor list already marshalled into a C array of ``gws_tensor``.

    The buffers of a training run do not move between steps, so the array can be
    built once with :func:`pack` and passed to every forward / backward call."""

    def __init__(self, arr, n, keepalive):
        self.arr, self.n, self._keepalive = arr, n, keepalive

    def __len__(self):
        return self.n


def pack(descs: Sequence[TensorDesc]) -> PackedTensors:
    return PackedTensors(_marshal(descs), len(descs), list(descs))


def _as_c(t):
    if isinstance(t, PackedTensors):
        return t.arr, t.n
    return _marshal(t), len(t)


def _marshal(descs: Sequence[TensorDesc]):
    arr = (_CTensor * max(1, len(descs)))()
    for c, d in zip(arr, descs):
        ld = d.ld
        if ld is None:
            ref = next((t for t in (d.w, d.g, d.dw) if t is not None), None)
            ld = int(ref.stride(0)) if ref is not None and ref.dim() == 2 else d.cols
        c.w, c.w_hat, c.bt, c.scale = _p(d.w), _p(d.w_hat), _p(d.bt), _p(d.scale)
        c.g, c.dw, c.dbt = _p(d.g), _p(d.dw), _p(d.dbt)
        c.rows, c.cols, c.ld, c.row0, c.col0 = d.rows, d.cols, ld, d.row0, d.col0
        c.seed = d.seed & (2 ** 64 - 1)
    return arr


def _check(rc: int, what: str):
    if rc != 0:
        raise GwsError(rc, what)


def gws_sample_fwd(t: Sequence[TensorDesc], fmt: int, step: int, stream=None) -> None:
    """Paper Eq. 3 + cast for every descriptor; writes ``w_hat`` and ``scale``."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_sample_fwd(arr, n, int(fmt), int(step), _stream(stream)), "gws_sample_fwd")


def gws_sample_bwd(t: Sequence[TensorDesc], step: int, stream=None) -> None:
    """Paper Eq. 4 for every descriptor; writes ``dbt`` (and ``dw`` unless aliased)."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_sample_bwd(arr, n, int(step), _stream(stream)), "gws_sample_bwd")


class PackedBitwidth:
    """Bitwidth settings already marshalled into a C array of ``gws_bitwidth`` (see :func:`pack_bitwidth`)."""

    def __init__(self, arr, n):
        self.arr, self.n = arr, n

    def __len__(self):
        return self.n


def pack_bitwidth(bw: Sequence[Bitwidth]) -> PackedBitwidth:
    arr = (_CBitwidth * max(1, len(bw)))()
    for c, b in zip(arr, bw):
        c.b_init, c.b_target, c.lam, c.layer_blocks = b.b_init, b.b_target, b.lam, b.layer_blocks
    return PackedBitwidth(arr, len(bw))


def _marshal_bw(bw, n: int):
    if len(bw) != n:
        raise ValueError(f"{n} tensors but {len(bw)} bitwidth settings")
    return (bw if isinstance(bw, PackedBitwidth) else pack_bitwidth(bw)).arr


def gws_sample_fwd_bi(t: Sequence[TensorDesc], bw: Sequence[Bitwidth], fmt: int, step: int, stream=None) -> None:
    """``gws_sample_fwd`` with ``bt`` holding the internal parameter b_i of paper Eq. 11."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_sample_fwd_bi(arr, n, _marshal_bw(bw, n), int(fmt), int(step), _stream(stream)),
           "gws_sample_fwd_bi")


def gws_sample_bwd_bi(t: Sequence[TensorDesc], bw: Sequence[Bitwidth], step: int, stream=None) -> None:
    """``gws_sample_bwd`` writing dL'/db_i (paper Eq. 11, Eq. 12) into ``dbt``; needs ``bt`` = b_i."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_sample_bwd_bi(arr, n, _marshal_bw(bw, n), int(step), _stream(stream)), "gws_sample_bwd_bi")


class PackedMxOut:
    """MX output descriptors already marshalled into a C array of ``gws_mx_out`` (see :func:`pack_mx`)."""

    def __init__(self, arr, n, keepalive):
        self.arr, self.n, self._keepalive = arr, n, keepalive

    def __len__(self):
        return self.n


def pack_mx(outs: Sequence[MxOut]) -> PackedMxOut:
    arr = (_CMxOut * max(1, len(outs)))()
    for c, o in zip(arr, outs):
        ldc = o.ldc
        if ldc is None:
            ldc = int(o.codes.stride(0)) if o.codes is not None and o.codes.dim() == 2 else 0
        c.codes, c.xscale, c.ldc = _p(o.codes), _p(o.xscale), ldc
    return PackedMxOut(arr, len(outs), list(outs))


def gws_sample_fwd_mx(t: Sequence[TensorDesc], o: Sequence[MxOut], fmt: int, step: int, stream=None) -> None:
    """``gws_sample_fwd`` writing MX element codes and E8M0 block scales instead of ``w_hat``."""
    L = load_library()
    arr, n = _as_c(t)
    if len(o) != n:
        raise ValueError(f"{n} tensors but {len(o)} MX outputs")
    oa = (o if isinstance(o, PackedMxOut) else pack_mx(o)).arr
    _check(L.gws_sample_fwd_mx(arr, oa, n, int(fmt), int(step), _stream(stream)), "gws_sample_fwd_mx")


def gws_linear_fwd(x, w: TensorDesc, y, fmt: int, step: int, w_is_nk: bool = False, stream=None) -> None:
    """Y = X * w_hat, the weight sampled as in ``gws_sample_fwd``; the library picks the faster of its two ways."""
    L = load_library()
    M, K = int(x.shape[0]), int(x.shape[1])
    _check(L.gws_linear_fwd(_p(x), M, K, int(x.stride(0)), _marshal([w]), int(bool(w_is_nk)), int(fmt),
                            int(step), _p(y), int(y.stride(0)), _stream(stream)), "gws_linear_fwd")


def gws_linear_fwd_mode(x, w: TensorDesc, y, fmt: int, step: int, mode: int, w_is_nk: bool = False, stream=None) -> None:
    """``gws_linear_fwd`` with the kernel choice made by the caller (``LINEAR_*``)."""
    L = load_library()
    M, K = int(x.shape[0]), int(x.shape[1])
    _check(L.gws_linear_fwd_mode(_p(x), M, K, int(x.stride(0)), _marshal([w]), int(bool(w_is_nk)), int(fmt),
                                 int(step), _p(y), int(y.stride(0)), int(mode), _stream(stream)), "gws_linear_fwd_mode")


def gws_linear_fwd_workspace_bytes(w: TensorDesc) -> int:
    """Bytes of device workspace ``gws_linear_fwd_ws`` needs for this weight."""
    return int(load_library().gws_linear_fwd_workspace_bytes(_marshal([w])))


def gws_linear_fwd_ws(x, w: TensorDesc, y, fmt: int, step: int, workspace, w_is_nk: bool = False, stream=None) -> None:
    """``gws_linear_fwd`` with w_hat and scale staged in ``workspace`` (a uint8 device tensor) instead of the caller's buffers."""
    L = load_library()
    M, K = int(x.shape[0]), int(x.shape[1])
    _check(L.gws_linear_fwd_ws(_p(x), M, K, int(x.stride(0)), _marshal([w]), int(bool(w_is_nk)), int(fmt), int(step),
                               _p(y), int(y.stride(0)), _p(workspace), int(workspace.numel() * workspace.element_size()),
                               _stream(stream)), "gws_linear_fwd_ws")


STATIC_SCRATCH_BYTES = 32 << 20


def gws_linear_fwd_static(x, w: TensorDesc, y, fmt: int, step: int, w_is_nk: bool = False, stream=None) -> None:
    """``gws_linear_fwd_ws`` without a workspace and without any allocation: w_hat is staged in the library's own buffer."""
    L = load_library()
    M, K = int(x.shape[0]), int(x.shape[1])
    _check(L.gws_linear_fwd_static(_p(x), M, K, int(x.stride(0)), _marshal([w]), int(bool(w_is_nk)), int(fmt), int(step),
                                   _p(y), int(y.stride(0)), _stream(stream)), "gws_linear_fwd_static")


def gws_linear_bwd_w(x, dy, w: TensorDesc, step: int, w_is_nk: bool = False, stream=None) -> None:
    """dW = X^T dY into ``w.dw`` and, when ``w.dbt`` is given, dL/db_t (paper Eq. 4) from the GEMM's epilogue."""
    L = load_library()
    _check(L.gws_linear_bwd_w(_p(x), _p(dy), int(x.shape[0]), int(x.stride(0)), int(dy.stride(0)), _marshal([w]),
                              int(bool(w_is_nk)), int(step), _stream(stream)), "gws_linear_bwd_w")


def gws_linear_bwd_w_workspace_bytes(w: TensorDesc, M: int) -> int:
    """Bytes ``gws_linear_bwd_w_ws`` would use for this weight over ``M`` tokens (0: the one-kernel form)."""
    L = load_library()
    return int(L.gws_linear_bwd_w_workspace_bytes(_marshal([w]), int(M)))


def gws_linear_bwd_w_ws(x, dy, w: TensorDesc, step: int, workspace, w_is_nk: bool = False, stream=None) -> None:
    """``gws_linear_bwd_w`` with the tokens split into parts through ``workspace`` (a device tensor, or None)."""
    L = load_library()
    nbytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    _check(L.gws_linear_bwd_w_ws(_p(x), _p(dy), int(x.shape[0]), int(x.stride(0)), int(dy.stride(0)), _marshal([w]),
                                 int(bool(w_is_nk)), int(step), _p(workspace), nbytes, _stream(stream)), "gws_linear_bwd_w_ws")


def gws_gemm_bf16(x, w, y, w_is_nk: bool = False, stream=None) -> None:
    """Plain BF16 GEMM twin of ``gws_linear_fwd`` (no sampling)."""
    L = load_library()
    M, K = int(x.shape[0]), int(x.shape[1])
    N = int(w.shape[0] if w_is_nk else w.shape[1])
    _check(L.gws_gemm_bf16(_p(x), M, K, int(x.stride(0)), _p(w), N, int(w.stride(0)), int(bool(w_is_nk)),
                           _p(y), int(y.stride(0)), _stream(stream)), "gws_gemm_bf16")


def gws_gemm_bf16_sample_next(x, w, y, nxt: Optional[TensorDesc], fmt: int, step: int, w_is_nk: bool = False, stream=None) -> None:
    """``gws_gemm_bf16`` with ``gws_sample_fwd([nxt], fmt, step)`` riding along in the same launch where that pays."""
    L = load_library()
    M, K = int(x.shape[0]), int(x.shape[1])
    N = int(w.shape[0] if w_is_nk else w.shape[1])
    arr = None if nxt is None else _marshal([nxt])
    _check(L.gws_gemm_bf16_sample_next(_p(x), M, K, int(x.stride(0)), _p(w), N, int(w.stride(0)), int(bool(w_is_nk)),
                                       _p(y), int(y.stride(0)), arr, int(fmt), int(step), _stream(stream)),
           "gws_gemm_bf16_sample_next")


def gws_gemm_bf16_sample_next_n(x, w, y, nxt, fmt: int, step: int, w_is_nk: bool = False, stream=None) -> None:
    """``gws_gemm_bf16`` with ``gws_sample_fwd(nxt, fmt, step)`` of a list of weights riding along where that pays."""
    L = load_library()
    M, K = int(x.shape[0]), int(x.shape[1])
    N = int(w.shape[0] if w_is_nk else w.shape[1])
    arr, n = _as_c(nxt)
    _check(L.gws_gemm_bf16_sample_next_n(_p(x), M, K, int(x.stride(0)), _p(w), N, int(w.stride(0)), int(bool(w_is_nk)),
                                         _p(y), int(y.stride(0)), arr, n, int(fmt), int(step), _stream(stream)),
           "gws_gemm_bf16_sample_next_n")


def gws_ride_plan(M: int, K: int, N: int, nxt) -> int:
    """How many of ``nxt`` would ride in the launch of an M x K x N GEMM (a measurement aid)."""
    arr, n = _as_c(nxt)
    return int(load_library().gws_ride_plan(int(M), int(K), int(N), arr, n))


def gws_gemm_bf16_ride_probe(x, w, y, nxt: TensorDesc, fmt: int, step: int, extra_workgroups: int, rider: int = 1,
                             w_is_nk: bool = False, stream=None) -> None:
    """``gws_gemm_bf16_sample_next`` with the riding forced (a measurement aid); ``x=None`` launches the riders alone."""
    L = load_library()
    if x is None:
        M = K = N = ldx = ldw = ldy = 0
    else:
        M, K = int(x.shape[0]), int(x.shape[1])
        N = int(w.shape[0] if w_is_nk else w.shape[1])
        ldx, ldw, ldy = int(x.stride(0)), int(w.stride(0)), int(y.stride(0))
    _check(L.gws_gemm_bf16_ride_probe(_p(x), M, K, ldx, _p(w), N, ldw, int(bool(w_is_nk)), _p(y), ldy, _marshal([nxt]),
                                      int(fmt), int(step), int(extra_workgroups), int(rider), _stream(stream)),
           "gws_gemm_bf16_ride_probe")


def gws_copy_tiles(t: Sequence[TensorDesc], stream=None) -> None:
    """Copy ``w`` to ``w_hat`` with the forward pass's access pattern (a measurement aid)."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_copy_tiles(arr, n, _stream(stream)), "gws_copy_tiles")


def gws_sample_bwd_tuned(t: Sequence[TensorDesc], step: int, variant: int = -1, per_x: int = 0, stream=None) -> None:
    """``gws_sample_bwd`` with the kernel variant and the column tiles per workgroup chosen by the caller (a measurement aid)."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_sample_bwd_tuned(arr, n, int(step), int(variant), int(per_x), _stream(stream)), "gws_sample_bwd_tuned")


def gws_sample_fwd_tuned(t: Sequence[TensorDesc], fmt: int, step: int, variant: int = -1, per_x: int = 0, stream=None) -> None:
    """``gws_sample_fwd`` with the kernel variant and the column tiles per workgroup chosen by the caller (a measurement aid)."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_sample_fwd_tuned(arr, n, int(fmt), int(step), int(variant), int(per_x), _stream(stream)), "gws_sample_fwd_tuned")


def gws_block_absmax(t: Sequence[TensorDesc], stream=None) -> None:
    """``scale`` := max|w| per 32x32 block (step one of paper Eq. 3; also the read-only ceiling measurement)."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_block_absmax(arr, n, _stream(stream)), "gws_block_absmax")


def gws_sample_fwd_basis(t: Sequence[TensorDesc], basis: int, fmt: int, step: int, stream=None) -> None:
    """``gws_sample_fwd`` with R drawn from a comparison basis (``BASIS_*``; paper Sec. 4)."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_sample_fwd_basis(arr, n, int(basis), int(fmt), int(step), _stream(stream)), "gws_sample_fwd_basis")


def gws_sample_bwd_basis(t: Sequence[TensorDesc], basis: int, step: int, stream=None) -> None:
    """``gws_sample_bwd`` with R drawn from a comparison basis."""
    L = load_library()
    arr, n = _as_c(t)
    _check(L.gws_sample_bwd_basis(arr, n, int(basis), int(step), _stream(stream)), "gws_sample_bwd_basis")


def gws_noise_basis(out, rows: int, cols: int, seed: int, step: int, basis: int, row0: int = 0, col0: int = 0,
                    stream=None) -> None:
    """R of a comparison basis as BF16 values into ``out`` [rows, cols]."""
    L = load_library()
    _check(L.gws_noise_basis(_p(out), rows, cols, row0, col0, seed & (2 ** 64 - 1), int(step), int(basis),
                             _stream(stream)), "gws_noise_basis")


def gws_noise_packed(out, rows: int, cols: int, seed: int, step: int, row0: int = 0, col0: int = 0,
                     stream=None) -> None:
    """Packed sign-magnitude noise codes, 8 per 32-bit word (paper Sec. 3.4)."""
    L = load_library()
    _check(L.gws_noise_packed(_p(out), rows, cols, row0, col0, seed & (2 ** 64 - 1), int(step),
                              _stream(stream)), "gws_noise_packed")


def gws_derive_seed(user_seed: int, tensor_id: int) -> int:
    return int(load_library().gws_derive_seed(user_seed & (2 ** 64 - 1), tensor_id & (2 ** 64 - 1)))


derive_seed = gws_derive_seed
