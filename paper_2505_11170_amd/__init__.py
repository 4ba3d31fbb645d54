"""GaussWS (Gaussian weight sampling) hot path for MI355X / gfx950.

Thin ctypes binding over ``libgws.so`` (hand-written HIP kernels behind a C ABI).
Importing the package does not load the library; calling any operation does, and
raises if the library has not been built.  There is no CPU fallback.
"""
from . import synth  # noqa: F401
from .binding import (  # noqa: F401
    BASIS_BITS, BASIS_BOX_MULLER, BASIS_UNIFORM_BF16, FMT_BF16, FMT_FP8_E4M3, FMT_FP6_E3M2, LINEAR_AUTO, LINEAR_IN_OPERAND, LINEAR_TWO_KERNELS, Bitwidth, GwsError, MxOut, PackedBitwidth, PackedMxOut, PackedTensors, STATIC_SCRATCH_BYTES, TensorDesc, derive_seed,
    gws_block_absmax, gws_copy_tiles, gws_derive_seed, gws_gemm_bf16, gws_gemm_bf16_ride_probe, gws_gemm_bf16_sample_next, gws_gemm_bf16_sample_next_n, gws_linear_bwd_w, gws_linear_bwd_w_workspace_bytes, gws_linear_bwd_w_ws, gws_linear_fwd, gws_linear_fwd_mode, gws_linear_fwd_static, gws_linear_fwd_workspace_bytes, gws_linear_fwd_ws, gws_noise_basis, gws_ride_plan, gws_noise_packed, gws_sample_bwd_basis, gws_sample_bwd_tuned, gws_sample_fwd_basis, gws_sample_bwd, gws_sample_bwd_bi,
    gws_sample_fwd, gws_sample_fwd_bi, gws_sample_fwd_mx, gws_sample_fwd_tuned, library_path, load_library, pack, pack_bitwidth, pack_mx,
)
