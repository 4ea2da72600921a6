"""Thin Python binding of the C ABI in include/cocktail.h.

Same names as the C entry points; this layer only marshals arguments.  torch is
used for device memory and for the current HIP stream, nothing else: every step
of the path (planning, reordering, quantisation, attention, merge) runs inside
libcocktail.so.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import _lib
from ._lib import Cache, CocktailError, Shape, Sizes, check, lib  # noqa: F401


def make_shape(batch: int, num_q_heads: int, num_kv_heads: int, head_dim: int, chunk_size: int,
               group_size: int) -> Shape:
    return Shape(batch, num_q_heads, num_kv_heads, head_dim, chunk_size, group_size)


@dataclass
class Plan:
    shape: Shape
    sizes: Sizes
    blob: np.ndarray            # uint8 [plan_bytes], host
    class_tokens: np.ndarray    # int32 [B, 4]: INT2, INT4, INT8, FP16
    perm: np.ndarray            # int32 [total_chunks]
    seq_lens: np.ndarray


def cocktail_default_workers(shape: Shape, vector_alu_only: bool = False) -> int:
    """Decode workgroups that fill the GPU for this shape (vector_alu_only: for a plan made with that option,
    where every workgroup is one wave whatever Hq/Hkv is)."""
    n = C.c_int32(0)
    if vector_alu_only:
        shape = Shape(shape.batch, shape.num_q_heads, shape.num_q_heads, shape.head_dim, shape.chunk_size, shape.group_size)
    check(lib().cocktail_default_workers(C.byref(shape), C.byref(n)))
    return int(n.value)


def cocktail_plan(shape: Shape, seq_lens: Sequence[int], chunk_bits: Sequence[int], num_workers: int,
                  append_capacity: int = 0, reproducible: bool = False, vector_alu_only: bool = False,
                  max_seq_lens: Optional[Sequence[int]] = None) -> Plan:
    """Host-only: Alg. 1's prefill partition plus cache layout and decode work split (cocktail_plan_ex).

    append_capacity > 0 reserves room for that many generated tokens per sequence; reproducible=True
    asks for a purely static decode split (bitwise identical results from call to call); vector_alu_only=True
    plans grouped-query shapes for the kernel without matrix instructions (one query head per wave);
    max_seq_lens lays the FP16 runs out with room to grow to those context lengths (cocktail_fold_appended).
    """
    sl = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    cb = np.ascontiguousarray(np.asarray(chunk_bits, dtype=np.uint8).reshape(-1))
    if sl.shape != (shape.batch,):
        raise ValueError("seq_lens must have one entry per sequence")
    need = int(sum(int(t) // shape.chunk_size for t in sl if t >= 0)) if shape.chunk_size > 0 else 0
    if cb.size != need:
        raise ValueError(f"chunk_bits has {cb.size} entries, {need} expected")
    sizes = Sizes()
    slp = sl.ctypes.data_as(C.POINTER(C.c_int32))
    cbp = cb.ctypes.data_as(C.POINTER(C.c_uint8)) if cb.size else None
    opt = _lib.PlanOptions(int(append_capacity), int(bool(reproducible)), int(bool(vector_alu_only)))
    if max_seq_lens is not None:
        ml = np.ascontiguousarray(np.asarray(max_seq_lens, dtype=np.int32))
        if ml.shape != (shape.batch,):
            raise ValueError("max_seq_lens must have one entry per sequence")
        opt.max_seq_lens = ml.ctypes.data_as(C.POINTER(C.c_int32))   # `ml` stays alive until both calls below return
    check(lib().cocktail_plan_ex(C.byref(shape), slp, cbp, num_workers, C.byref(opt), C.byref(sizes), None, 0, None,
                                 None))
    blob = np.zeros(int(sizes.plan_bytes), dtype=np.uint8)
    ct = np.zeros((shape.batch, _lib.NUM_CLASSES), dtype=np.int32)
    perm = np.zeros(max(int(sizes.total_chunks), 1), dtype=np.int32)
    check(lib().cocktail_plan_ex(C.byref(shape), slp, cbp, num_workers, C.byref(opt), C.byref(sizes),
                                 blob.ctypes.data, blob.size, ct.ctypes.data_as(C.POINTER(C.c_int32)),
                                 perm.ctypes.data_as(C.POINTER(C.c_int32))))
    return Plan(shape, sizes, blob, ct, perm[:int(sizes.total_chunks)], sl)


def cocktail_plan_field(plan: Plan, name: str, index: int = 0) -> int:
    """Debugging aid: one field of the plan's internal header, by its name in the library's source."""
    v = C.c_int64(0)
    check(lib().cocktail_plan_field(plan.blob.ctypes.data, name.encode(), int(index), C.byref(v)))
    return int(v.value)


class PackedCache:
    """Device buffers of one layer's packed cache plus the ctypes descriptor handed to the library."""

    def __init__(self, plan: Plan, device: torch.device):
        self.plan = plan
        self.device = device
        self.plan_dev = torch.from_numpy(plan.blob).to(device)
        self.k: List[torch.Tensor] = []
        self.v: List[torch.Tensor] = []
        for c in range(_lib.NUM_CLASSES):
            n = int(plan.sizes.class_bytes[c])
            self.k.append(torch.empty(n, dtype=torch.uint8, device=device))
            self.v.append(torch.empty(n, dtype=torch.uint8, device=device))
        self.desc = Cache()
        for c in range(_lib.NUM_CLASSES):
            self.desc.k[c] = self.k[c].data_ptr() if self.k[c].numel() else None
            self.desc.v[c] = self.v[c].data_ptr() if self.v[c].numel() else None
        self.desc.plan_host = plan.blob.ctypes.data
        self.desc.plan_dev = self.plan_dev.data_ptr()
        nb = int(plan.sizes.append_bytes)
        self.k_app = torch.empty(nb, dtype=torch.uint8, device=device) if nb else None
        self.v_app = torch.empty(nb, dtype=torch.uint8, device=device) if nb else None
        self.desc.k_app = self.k_app.data_ptr() if nb else None
        self.desc.v_app = self.v_app.data_ptr() if nb else None
        self.desc.num_appended = 0
        # per-sequence counts of appended tokens, used once cocktail_append_fp16_ragged is called (NULL before:
        # lockstep batches count in desc.num_appended)
        self.appended = torch.zeros(plan.shape.batch, dtype=torch.int32, device=device) if nb else None
        self.desc.appended_dev = None
        self.workspace = torch.empty(int(plan.sizes.workspace_bytes), dtype=torch.uint8, device=device)


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def cocktail_reorder_quantize(cache: PackedCache, k_src: torch.Tensor, v_src: torch.Tensor, *,
                              ragged: bool = False, stride_b: int = 0, stride_h: int = 0,
                              stride_t: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Reorder + quantise + pack K and V (device fp16 tensors) into `cache`.

    Strided layout: element (b,h,t,d) at b*stride_b + h*stride_h + t*stride_t + d.  With ragged=True the
    sequences are concatenated, each stored as [Hkv][T_b] rows of stride_t elements.
    """
    if k_src.dtype != torch.float16 or v_src.dtype != torch.float16:
        raise TypeError("k_src and v_src must be float16")
    if not (k_src.is_cuda and v_src.is_cuda):
        raise ValueError("k_src and v_src must be device tensors")
    sh = cache.plan.shape
    st = sh.head_dim if stride_t is None else stride_t
    if not ragged and stride_b == 0 and stride_h == 0:
        # no strides given: a contiguous [B, Hkv, T, stride_t] tensor
        if k_src.dim() != 4 or not k_src.is_contiguous() or k_src.shape != v_src.shape or k_src.shape[:2] != (sh.batch, sh.num_kv_heads):
            raise ValueError("without strides k_src and v_src must be contiguous [B, Hkv, T, D] tensors")
        st = int(k_src.stride(2)) if stride_t is None else st
        stride_b, stride_h = int(k_src.stride(0)), int(k_src.stride(1))
    check(lib().cocktail_reorder_quantize(C.byref(sh), k_src.data_ptr(), v_src.data_ptr(),
                                          _lib.SRC_RAGGED if ragged else _lib.SRC_STRIDED, stride_b, stride_h, st,
                                          C.byref(cache.desc), _stream_ptr(stream)))


def cocktail_reorder_quantize_paged(cache: PackedCache, k_pages: torch.Tensor, v_pages: torch.Tensor,
                                    page_table: torch.Tensor, *, head_major: bool = True,
                                    stream: Optional[torch.cuda.Stream] = None) -> None:
    """Reorder + quantise + pack from a paged KV cache.  k_pages, v_pages: device fp16 [num_pages, Hkv, page_size, D]
    (head_major) or [num_pages, page_size, Hkv, D]; page_table: device int32 [B, max pages per sequence]."""
    sh = cache.plan.shape
    for t in (k_pages, v_pages):
        if t.dtype != torch.float16 or not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise TypeError("k_pages and v_pages must be contiguous 4-d float16 device tensors")
    if k_pages.shape != v_pages.shape or k_pages.shape[3] != sh.head_dim:
        raise ValueError("k_pages and v_pages must have the same shape [pages, ., ., D]")
    if page_table.dtype != torch.int32 or not page_table.is_cuda or not page_table.is_contiguous() or page_table.dim() != 2:
        raise TypeError("page_table must be a contiguous int32 device tensor [B, pages per sequence]")
    if page_table.shape[0] != sh.batch:
        raise ValueError("page_table needs one row per sequence")
    num_pages, a, b, d = k_pages.shape
    page_size, hkv = (b, a) if head_major else (a, b)
    if hkv != sh.num_kv_heads:
        raise ValueError("page pools do not hold num_kv_heads heads")
    src = _lib.PagedSource(k_pages.data_ptr(), v_pages.data_ptr(), page_table.data_ptr(), int(page_table.shape[1]),
                           int(page_size), int(num_pages), 0, int(k_pages.stride(0)),
                           int(k_pages.stride(1 if head_major else 2)), int(k_pages.stride(2 if head_major else 1)))
    check(lib().cocktail_reorder_quantize_paged(C.byref(sh), C.byref(src), C.byref(cache.desc), _stream_ptr(stream)))


def cocktail_append_fp16(cache: PackedCache, k_new: torch.Tensor, v_new: torch.Tensor,
                         position: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Stores one generated token per sequence (device fp16 [B, Hkv, D]) as appended token `position`
    (default: the next free one) and makes the following decode calls attend to it."""
    sh = cache.plan.shape
    for t in (k_new, v_new):
        if t.dtype != torch.float16 or not t.is_cuda or not t.is_contiguous():
            raise TypeError("k_new and v_new must be contiguous float16 device tensors")
        if tuple(t.shape) != (sh.batch, sh.num_kv_heads, sh.head_dim):
            raise ValueError("k_new and v_new must have shape [B, Hkv, D]")
    pos = int(cache.desc.num_appended) if position is None else int(position)
    check(lib().cocktail_append_fp16(C.byref(sh), k_new.data_ptr(), v_new.data_ptr(), C.byref(cache.desc), pos,
                                     _stream_ptr(stream)))
    cache.desc.num_appended = max(int(cache.desc.num_appended), pos + 1)


def cocktail_append_fp16_ragged(cache: PackedCache, k_new: torch.Tensor, v_new: torch.Tensor,
                                active: Optional[torch.Tensor] = None,
                                stream: Optional[torch.cuda.Stream] = None) -> None:
    """Stores one generated token for every sequence with active[b] != 0 (device uint8 [B]; None = all) behind
    what that sequence has appended so far and advances its count (cache.appended, on the device)."""
    sh = cache.plan.shape
    for t in (k_new, v_new):
        if t.dtype != torch.float16 or not t.is_cuda or not t.is_contiguous():
            raise TypeError("k_new and v_new must be contiguous float16 device tensors")
        if tuple(t.shape) != (sh.batch, sh.num_kv_heads, sh.head_dim):
            raise ValueError("k_new and v_new must have shape [B, Hkv, D]")
    if active is not None and (active.dtype != torch.uint8 or not active.is_cuda or tuple(active.shape) != (sh.batch,)):
        raise TypeError("active must be a uint8 device tensor [B]")
    if cache.appended is None:
        raise ValueError("the plan was made without append buffers")
    if int(cache.desc.num_appended) != 0:
        raise ValueError("this cache counts appended tokens in lockstep (cocktail_append_fp16); do not mix the two")
    cache.desc.appended_dev = cache.appended.data_ptr()
    check(lib().cocktail_append_fp16_ragged(C.byref(sh), k_new.data_ptr(), v_new.data_ptr(), C.byref(cache.desc),
                                            active.data_ptr() if active is not None else None, _stream_ptr(stream)))


def cocktail_fold_appended(cache: PackedCache, new_plan: Plan, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Moves the appended tokens of every sequence into the packed cache (they become context) and switches the
    cache to `new_plan`, the plan of the longer contexts made with the same max_seq_lens."""
    sh = cache.plan.shape
    s = stream if stream is not None else torch.cuda.current_stream()
    with torch.cuda.stream(s):
        new_dev = torch.from_numpy(new_plan.blob).to(cache.device)       # stream-ordered before the fold
        check(lib().cocktail_fold_appended(C.byref(sh), C.byref(cache.desc), new_plan.blob.ctypes.data, new_dev.data_ptr(),
                                           _stream_ptr(s)))
        old_dev = cache.plan_dev
        old_dev.record_stream(s)
        if int(new_plan.sizes.workspace_bytes) > cache.workspace.numel():
            cache.workspace.record_stream(s)
            cache.workspace = torch.empty(int(new_plan.sizes.workspace_bytes), dtype=torch.uint8, device=cache.device)
    cache.plan, cache.plan_dev = new_plan, new_dev
    cache.desc.plan_host = new_plan.blob.ctypes.data
    cache.desc.plan_dev = new_dev.data_ptr()
    cache.desc.num_appended = 0


def cocktail_decode_attention(cache: PackedCache, q: torch.Tensor, sm_scale: float = 0.0,
                              out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                              stream: Optional[torch.cuda.Stream] = None):
    """Single-query attention over the packed cache.  q: device fp16 [B, Hq, D].  Returns (out, lse)."""
    sh = cache.plan.shape
    if q.dtype != torch.float16 or not q.is_cuda or not q.is_contiguous():
        raise TypeError("q must be a contiguous float16 device tensor")
    if tuple(q.shape) != (sh.batch, sh.num_q_heads, sh.head_dim):
        raise ValueError("q must have shape [B, Hq, D]")
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((sh.batch, sh.num_q_heads), dtype=torch.float32, device=q.device)
    check(lib().cocktail_decode_attention(C.byref(sh), q.data_ptr(), C.byref(cache.desc), float(sm_scale),
                                          out.data_ptr(), lse.data_ptr(), cache.workspace.data_ptr(),
                                          cache.workspace.numel(), _stream_ptr(stream)))
    return out, lse


def cocktail_decode_attention_marked(cache: PackedCache, q: torch.Tensor, event_between: torch.cuda.Event,
                                     out: torch.Tensor, lse: torch.Tensor, sm_scale: float = 0.0,
                                     stream: Optional[torch.cuda.Stream] = None) -> None:
    """Measurement aid: cocktail_decode_attention that records `event_between` (created with enable_timing=True
    and recorded once before, so that its handle exists) between the partial-state kernel and the merge."""
    handle = int(event_between.cuda_event)
    if not handle:
        raise ValueError("record event_between once before passing it, torch creates the handle lazily")
    check(lib().cocktail_decode_attention_marked(C.byref(cache.plan.shape), q.data_ptr(), C.byref(cache.desc), float(sm_scale),
                                                 out.data_ptr(), lse.data_ptr(), cache.workspace.data_ptr(),
                                                 cache.workspace.numel(), _stream_ptr(stream), handle))


def cocktail_decode_attention_static(cache: PackedCache, q: torch.Tensor, sm_scale: float, out: torch.Tensor,
                                     lse: Optional[torch.Tensor] = None,
                                     stream: Optional[torch.cuda.Stream] = None) -> None:
    """cocktail_decode_attention on the workspace built into the library: nothing is allocated, so the caller
    passes `out` (and `lse`, if wanted)."""
    sh = cache.plan.shape
    if q.dtype != torch.float16 or not q.is_cuda or not q.is_contiguous():
        raise TypeError("q must be a contiguous float16 device tensor")
    if tuple(q.shape) != (sh.batch, sh.num_q_heads, sh.head_dim) or out.shape != q.shape or out.dtype != q.dtype:
        raise ValueError("q and out must be float16 [B, Hq, D]")
    check(lib().cocktail_decode_attention_static(C.byref(sh), q.data_ptr(), C.byref(cache.desc), float(sm_scale),
                                                 out.data_ptr(), lse.data_ptr() if lse is not None else None,
                                                 _stream_ptr(stream)))


def cocktail_decode_check(cache: PackedCache, stream: Optional[torch.cuda.Stream] = None,
                          static_workspace: bool = False) -> None:
    """Waits for the stream and raises CocktailError (code -6) if the last decode call on this cache's
    workspace (or on the library's built-in one) did not attend to every token exactly once."""
    check(lib().cocktail_decode_check(C.byref(cache.plan.shape), C.byref(cache.desc),
                                      None if static_workspace else cache.workspace.data_ptr(), _stream_ptr(stream)))


def cocktail_stream_read_probe(buf: torch.Tensor, sink: torch.Tensor,
                               stream: Optional[torch.cuda.Stream] = None) -> int:
    """Enqueues a plain streaming read of `buf` (device, uint8); returns the bytes the launch reads."""
    if not (buf.is_cuda and sink.is_cuda and buf.is_contiguous()):
        raise ValueError("buf and sink must be contiguous device tensors")
    n = C.c_size_t(0)
    check(lib().cocktail_stream_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(),
                                           C.byref(n), _stream_ptr(stream)))
    return int(n.value)


def cocktail_chunk_bitwidths(query_emb: torch.Tensor, chunk_emb: torch.Tensor, num_chunks: Sequence[int],
                             alpha: float = 0.6, beta: float = 0.1, stream: Optional[torch.cuda.Stream] = None):
    """Chunk-level quantization search.  query_emb: device fp32 [B, E]; chunk_emb: device fp32 [sum N_b, E].
    Returns (chunk_bits uint8 [sum N_b], scores fp32 [sum N_b]), both on the device."""
    for t in (query_emb, chunk_emb):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
            raise TypeError("embeddings must be contiguous float32 device tensors")
    batch, e = query_emb.shape
    off = np.zeros(batch + 1, dtype=np.int32)
    off[1:] = np.cumsum(np.asarray(num_chunks, dtype=np.int64))
    total = int(off[-1])
    if chunk_emb.shape != (total, e) or len(num_chunks) != batch:
        raise ValueError("chunk_emb must have shape [sum(num_chunks), E] and num_chunks one entry per sequence")
    off_dev = torch.from_numpy(off).to(query_emb.device)
    scores = torch.empty(total, dtype=torch.float32, device=query_emb.device)
    bits = torch.empty(total, dtype=torch.uint8, device=query_emb.device)
    check(lib().cocktail_chunk_bitwidths(batch, e, total, off_dev.data_ptr(), query_emb.data_ptr(),
                                         chunk_emb.data_ptr() if total else None, float(alpha), float(beta),
                                         scores.data_ptr() if total else None, bits.data_ptr() if total else None,
                                         _stream_ptr(stream)))
    return bits, scores


def cocktail_selftest_arithmetic(device: torch.device, stream: Optional[torch.cuda.Stream] = None) -> List[int]:
    """Runs the exhaustive check of the quantizer's division shortcuts; returns the four mismatch counts
    (/ 3, / 15, 1 / scale, / 255)."""
    out = torch.empty(4, dtype=torch.int64, device=device)
    check(lib().cocktail_selftest_arithmetic(out.data_ptr(), _stream_ptr(stream)))
    return [int(x) for x in out.cpu().tolist()]
