"""MI355X-native W4A4 hot path of SingleQuant (arxiv 2511.22316): the online Givens + Kronecker
rotation fused with per-token int4 quantization, and the int4 x int4 GEMM with dequant epilogue.

``binding`` is the thin ctypes layer over the C-ABI library built from ``csrc/``;
``synth`` draws the seeded synthetic layers used by tests and the benchmark.
"""
from . import synth  # noqa: F401
from .binding import (  # noqa: F401
    SQError,
    library_path,
    sq_prepare_weights,
    sq_rotate_quantize,
    sq_w4a4_gemm,
    sq_status_string,
)
