"""MI355X (gfx950) native FlexiQ hot path: thin Python binding over libflexiq.so (C ABI in include/flexiq.h).

Argument marshalling only: every step runs in the HIP library.  PyTorch supplies device memory and
streams.  Importing this package never falls back to a CPU implementation: if the shared library
is missing, `load()` raises."""
from .binding import (FlexiqError, Layer, flexiq_bitlower, flexiq_dynamic_positions, flexiq_dynamic_positions_static, flexiq_static_positions,
                      flexiq_layer_positions, flexiq_input_prelowered, flexiq_layer_dump, flexiq_mixed_conv_implicit,
                      flexiq_mixed_gemm, flexiq_permute_channels, flexiq_quantize_act, flexiq_quantize_pack,
                      flexiq_set_ratio, exported_symbols, load, debug_force_tile, debug_force_packed4,
                      debug_max_blocks, debug_last_launch, flexiq_fp6_channels, flexiq_fp6_bytes, flexiq_lower_fp6,
                      flexiq_mixed_gemm_fp6, debug_force_fp6_tile,
                      flexiq_packed4_channels, flexiq_packed4_bytes, flexiq_lower_packed4, flexiq_mixed_gemm_packed4,
                      debug_force_stream, debug_force_conv3, debug_force_few_rows, debug_force_tile_splitk)

__all__ = ["FlexiqError", "Layer", "flexiq_bitlower", "flexiq_dynamic_positions", "flexiq_dynamic_positions_static", "flexiq_static_positions",
           "flexiq_layer_positions", "flexiq_input_prelowered", "flexiq_layer_dump", "flexiq_mixed_conv_implicit",
           "flexiq_mixed_gemm", "flexiq_permute_channels", "flexiq_quantize_act", "flexiq_quantize_pack",
           "flexiq_set_ratio", "exported_symbols", "load", "debug_force_tile", "debug_force_packed4", "debug_max_blocks", "debug_last_launch", "flexiq_fp6_channels", "flexiq_fp6_bytes", "flexiq_lower_fp6",
           "flexiq_mixed_gemm_fp6", "debug_force_fp6_tile",
           "flexiq_packed4_channels", "flexiq_packed4_bytes", "flexiq_lower_packed4", "flexiq_mixed_gemm_packed4",
           "debug_force_stream", "debug_force_conv3", "debug_force_few_rows", "debug_force_tile_splitk"]
