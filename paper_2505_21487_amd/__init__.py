"""MI355X-native GLA / GTA decode attention (hand-written HIP behind a C ABI).

`binding` wraps libgla_decode.so; `accounting` holds the byte / FLOP formulas
used for roofline reporting; `harness` uploads synthetic problems to the GPU.
"""
from .binding import (GLA_DECODE_NOALLOC_SCRATCH_BYTES, GLA_ERR_INVALID_ARG, GLA_ERR_LAUNCH, GLA_ERR_UNSUPPORTED_SHAPE,
                      GLA_ERR_WORKSPACE_TOO_SMALL, GLA_IMPL_AUTO, GLA_IMPL_GENERIC,
                      GLA_IMPL_TUNED, GLA_OK, GlaDecodeParams, GlaError, GlaProjParams, gla_absorb_query, gla_decode,
                      gla_decode_check_contents, gla_decode_noalloc, gla_decode_profile, gla_decode_select_impl, gla_decode_version,
                      gla_decode_workspace_size, gla_output_proj, gla_status_string, gqa_decode, gqa_decode_prepared, gta_decode, load_library,
                      make_params, shape_params, decode_prepared)

__all__ = [n for n in dir() if n.startswith(("gla_", "gta_", "gqa_", "GLA_", "Gla"))] + [
    "load_library", "make_params", "shape_params", "decode_prepared", "gqa_decode_prepared"]
