"""MI355X-native W4A4 hot path of SingleQuant (arxiv 2511.22316): the online Givens + Kronecker
rotation fused with per-token int4 quantization, the int4 x int4 GEMM with dequant epilogue, the
offline weight path and the closed-form construction of the rotation.

``binding`` is the thin ctypes layer over the C-ABI library built from ``csrc/``;
``synth`` draws the seeded synthetic layers used by tests and the benchmark.
"""
from . import synth  # noqa: F401
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    SQError,
    library_path,
    sq_build_rotation,
    sq_debug_set_option,
    sq_build_rotation_workspace_bytes,
    sq_decode_layer,
    sq_decode_layer_static,
    sq_decode_layer_status,
    sq_decode_layer_workspace_bytes,
    sq_kron_factor,
    sq_prepare_rotation,
    sq_pack_w3,
    sq_prepare_weights,
    sq_prepare_weights_variant,
    sq_prepared_rotation_bytes,
    sq_rotate_fp16,
    sq_rotate_quantize,
    sq_rotate_quantize_prepared,
    sq_rotate_quantize_variant,
    sq_w3a16_gemm,
    sq_w4a4_gemm,
    sq_w4a4_gemm_decode,
    sq_tile_weights_decode,
    sq_decode_weights_bytes,
    sq_w4a16_gemm,
    sq_status_string,
)
