"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds none of the method's arithmetic: only shapes and random draws.  The
shapes are the linear weights of the models the paper trains (GPT2-124M,
Llama2-style decoders; paper Sec. 4 and Fig. 6's layer order); the value
distributions stand in for trained weights and gradients, which are not
available: W ~ N(0, 0.02) (an init-like spread), the blockwise bitwidth b_t
constant or uniform in [4, 9] (the range Fig. 6 reports for >99 % of the
parameters), upstream dL/dw_hat ~ N(0, 1e-3), activations X ~ N(0, 1).

Tensor ``i`` of a workload draws from ``torch.Generator().manual_seed(1000 + i)``
in the fixed order W, b_t, g.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

BL = 32  # square block edge b_l


@dataclass(frozen=True)
class Shape:
    name: str
    rows: int
    cols: int


def gpt2_124m_shapes():
    """12 blocks x {qkv 768x2304, out 768x768, up 768x3072, down 3072x768}."""
    out = []
    for b in range(12):
        out += [Shape(f"h{b}.qkv", 768, 2304), Shape(f"h{b}.out", 768, 768),
                Shape(f"h{b}.up", 768, 3072), Shape(f"h{b}.down", 3072, 768)]
    return out


def llama_1b_shapes():
    """~1B Llama2-style decoder: hidden 2048, 22 layers, 32 q / 4 kv heads of dim 64,
    SwiGLU intermediate 5632; layer order (q, k, v, out, gate, down, up)."""
    out = []
    for l in range(22):
        out += [Shape(f"l{l}.q", 2048, 2048), Shape(f"l{l}.k", 256, 2048), Shape(f"l{l}.v", 256, 2048),
                Shape(f"l{l}.o", 2048, 2048), Shape(f"l{l}.gate", 5632, 2048),
                Shape(f"l{l}.down", 2048, 5632), Shape(f"l{l}.up", 5632, 2048)]
    return out


def n_blocks(rows: int, cols: int):
    return (rows + BL - 1) // BL, (cols + BL - 1) // BL


def _gen(index: int, device):
    g = torch.Generator(device=device)
    g.manual_seed(1000 + index)
    return g


def make_tensor(index: int, rows: int, cols: int, *, bt=None, device="cpu", with_grad=True,
                w_std=0.02, g_std=1e-3, ld=None):
    """Returns dict(w=BF16 [rows, ld], bt=fp32 [nbr, nbc], g=BF16 [rows, ld] or None).

    ``bt``: None -> uniform in [4, 9]; a float -> that constant for every block.
    ``ld`` > cols pads each row (padding is drawn like the data)."""
    ld = cols if ld is None else ld
    gen = _gen(index, device)
    w = (torch.randn(rows, ld, generator=gen, device=device, dtype=torch.float32) * w_std).to(torch.bfloat16)
    nbr, nbc = n_blocks(rows, cols)
    u = torch.rand(nbr, nbc, generator=gen, device=device, dtype=torch.float32)
    if bt is None:
        btt = 4.0 + 5.0 * u
    else:
        btt = torch.full((nbr, nbc), float(bt), device=device, dtype=torch.float32)
    g = None
    if with_grad:
        g = (torch.randn(rows, ld, generator=gen, device=device, dtype=torch.float32) * g_std).to(torch.bfloat16)
    return {"w": w, "bt": btt, "g": g}


def make_activation(index: int, m: int, k: int, device="cpu"):
    gen = _gen(index, device)
    return torch.randn(m, k, generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)


def bits(t: torch.Tensor):
    """BF16 tensor -> numpy uint16 bit patterns (host copy)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view("uint16")


def from_bits(a, device="cpu"):
    """numpy uint16 bit patterns -> BF16 tensor."""
    import numpy as np
    return torch.from_numpy(np.ascontiguousarray(a).view("int16")).view(torch.bfloat16).to(device)
