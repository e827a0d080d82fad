"""MI355X-native ReaLB rank layer: thin Python binding over the C-ABI library
librealb.so (hand-written HIP for gfx950).  PyTorch is used only for device
memory and streams; every step of the path runs in the library's kernels.
There is no CPU fallback: loading fails loudly if the library is not built."""
from .binding import (  # noqa: F401
    BF16, FP4, FORCE_NONE, RealbError, Config, Context, LayerBuffers, WeightBuffers, load_library,
    quantize_rows_fp4, quantize_rows_nvfp4, route_stats_static, amax_bf16, select_precision_host, bf16_from_bits, bits_from_bf16, library_path, scales_to_canonical,
)
