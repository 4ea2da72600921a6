"""MI355X-native chunk-level KV cache computation of Cocktail (arXiv 2503.23294, Sec. III-C).

The work is done by hand-written HIP kernels in libcocktail.so behind the C ABI
of include/cocktail.h; this package is the thin binding over it.
"""
from .api import (CocktailError, PackedCache, Plan, Shape, cocktail_append_fp16, cocktail_append_fp16_ragged, cocktail_chunk_bitwidths, cocktail_fold_appended,
                  cocktail_decode_attention, cocktail_decode_attention_marked, cocktail_decode_attention_static, cocktail_decode_check,
                  cocktail_default_workers, cocktail_plan_field,
                  cocktail_plan, cocktail_reorder_quantize, cocktail_reorder_quantize_paged, cocktail_selftest_arithmetic,
                  cocktail_stream_read_probe, make_shape)

__all__ = ["CocktailError", "PackedCache", "Plan", "Shape", "cocktail_append_fp16", "cocktail_append_fp16_ragged", "cocktail_chunk_bitwidths", "cocktail_fold_appended",
           "cocktail_decode_attention", "cocktail_decode_attention_marked", "cocktail_decode_attention_static", "cocktail_decode_check",
           "cocktail_default_workers", "cocktail_plan_field", "cocktail_plan", "cocktail_reorder_quantize", "cocktail_reorder_quantize_paged", "cocktail_selftest_arithmetic",
           "cocktail_stream_read_probe",
           "make_shape"]
