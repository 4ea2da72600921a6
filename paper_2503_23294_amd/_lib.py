"""ctypes loader for libcocktail.so (argument marshalling only).

`import torch` happens first on purpose: torch brings its own HIP runtime and
the library must bind to that one so that torch's streams and device pointers
are valid inside it.  There is no fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes as C
import os

import torch  # noqa: F401  (must be imported before the library is loaded)

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("COCKTAIL_LIB", os.path.join(HERE, "libcocktail.so"))

NUM_CLASSES = 4
TOKENS_PER_BLOCK = 64
MAX_Q_PER_KV = 64
STATIC_WORKSPACE_BYTES = 16 << 20

OK, EINVAL, EUNSUPPORTED, EALIGN, ENOSPACE, EHIP, ESTATE = 0, -1, -2, -3, -4, -5, -6
SRC_STRIDED, SRC_RAGGED = 0, 1


class Shape(C.Structure):
    _fields_ = [("batch", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("chunk_size", C.c_int32), ("group_size", C.c_int32)]


class Sizes(C.Structure):
    _fields_ = [("total_chunks", C.c_int64), ("class_tokens", C.c_int64 * NUM_CLASSES),
                ("class_blocks", C.c_int64 * NUM_CLASSES), ("class_bytes", C.c_int64 * NUM_CLASSES), ("plan_bytes", C.c_int64), ("workspace_bytes", C.c_int64),
                ("packed_bytes", C.c_int64), ("num_workers", C.c_int32), ("num_partials", C.c_int32),
                ("num_segments", C.c_int32), ("append_capacity", C.c_int32), ("append_bytes", C.c_int64),
                ("v_layout", C.c_int32), ("reserved", C.c_int32)]


class PlanOptions(C.Structure):
    _fields_ = [("append_capacity", C.c_int32), ("reproducible", C.c_int32), ("vector_alu_only", C.c_int32),
                ("reserved0", C.c_int32), ("max_seq_lens", C.POINTER(C.c_int32)), ("reserved", C.c_int32 * 2)]


class Cache(C.Structure):
    _fields_ = [("k", C.c_void_p * NUM_CLASSES), ("v", C.c_void_p * NUM_CLASSES), ("plan_host", C.c_void_p), ("plan_dev", C.c_void_p),
                ("k_app", C.c_void_p), ("v_app", C.c_void_p), ("num_appended", C.c_int32), ("reserved", C.c_int32),
                ("appended_dev", C.c_void_p)]


class PagedSource(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("page_table", C.c_void_p),
                ("table_stride", C.c_int32), ("page_size", C.c_int32), ("num_pages", C.c_int32), ("reserved", C.c_int32),
                ("stride_page", C.c_int64), ("stride_h", C.c_int64), ("stride_t", C.c_int64)]


EXPORTS = {
    "cocktail_plan": (C.c_int, [C.POINTER(Shape), C.POINTER(C.c_int32), C.POINTER(C.c_uint8), C.c_int32,
                                C.POINTER(Sizes), C.c_void_p, C.c_size_t, C.POINTER(C.c_int32),
                                C.POINTER(C.c_int32)]),
    "cocktail_plan_ex": (C.c_int, [C.POINTER(Shape), C.POINTER(C.c_int32), C.POINTER(C.c_uint8), C.c_int32,
                                   C.POINTER(PlanOptions), C.POINTER(Sizes), C.c_void_p, C.c_size_t,
                                   C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "cocktail_append_fp16": (C.c_int, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.POINTER(Cache), C.c_int32,
                                       C.c_void_p]),
    "cocktail_append_fp16_ragged": (C.c_int, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.POINTER(Cache), C.c_void_p,
                                              C.c_void_p]),
    "cocktail_fold_appended": (C.c_int, [C.POINTER(Shape), C.POINTER(Cache), C.c_void_p, C.c_void_p, C.c_void_p]),
    "cocktail_chunk_bitwidths": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_float, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]),
    "cocktail_reorder_quantize": (C.c_int, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_int32, C.c_int64,
                                            C.c_int64, C.c_int64, C.POINTER(Cache), C.c_void_p]),
    "cocktail_reorder_quantize_paged": (C.c_int, [C.POINTER(Shape), C.POINTER(PagedSource), C.POINTER(Cache), C.c_void_p]),
    "cocktail_decode_attention": (C.c_int, [C.POINTER(Shape), C.c_void_p, C.POINTER(Cache), C.c_float, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "cocktail_decode_attention_marked": (C.c_int, [C.POINTER(Shape), C.c_void_p, C.POINTER(Cache), C.c_float, C.c_void_p,
                                                   C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "cocktail_decode_attention_static": (C.c_int, [C.POINTER(Shape), C.c_void_p, C.POINTER(Cache), C.c_float,
                                                   C.c_void_p, C.c_void_p, C.c_void_p]),
    "cocktail_decode_check": (C.c_int, [C.POINTER(Shape), C.POINTER(Cache), C.c_void_p, C.c_void_p]),
    "cocktail_plan_field": (C.c_int, [C.c_void_p, C.c_char_p, C.c_int32, C.POINTER(C.c_int64)]),
    "cocktail_default_workers": (C.c_int, [C.POINTER(Shape), C.POINTER(C.c_int32)]),
    "cocktail_stream_read_probe": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_size_t), C.c_void_p]),
    "cocktail_selftest_arithmetic": (C.c_int, [C.c_void_p, C.c_void_p]),
    "cocktail_last_error": (C.c_char_p, []),
    "cocktail_version": (C.c_int, []),
}

_lib = None


class CocktailError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"cocktail error {code}: {message}")
        self.code = code


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2503_23294_amd.build` "
                "(there is no CPU or PyTorch fallback for the Cocktail kernels)")
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def check(rc: int) -> None:
    if rc != OK:
        raise CocktailError(rc, lib().cocktail_last_error().decode())
