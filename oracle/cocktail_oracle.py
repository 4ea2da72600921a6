"""CPU oracle for Cocktail's chunk-level KV cache computation (Sec. III-C, Algorithm 1).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, obviously-correct numpy
implementation that the tests, the smoke check and the bench's `cpu_baseline`
leg compare the HIP path against.  It shares no code with the HIP path and the
product never calls it.

What it computes, in the paper's order:
  plan            Alg. 1, prefill loop: every chunk goes to the list of its
                  bitwidth (INT2 / INT4 / FP16) in loop order; the remainder of
                  the context that does not fill a chunk stays FP16 (Sec. III-A).
  quantize_rows   Alg. 1 `quant` applied to the INT2 and INT4 lists.  The paper
                  names the function only; the reading used here is per-token
                  asymmetric min/max quantisation in groups of G channels along
                  head_dim with an fp16 scale and an fp16 zero (= group minimum).
  attention       Alg. 1, decode phase: logits of the three blocks concatenated
                  in the order INT2, INT4, FP16, one softmax over the
                  concatenation, three att x V products summed.  Evaluated in
                  float64 on the dequantised values.
  chunk_bitwidths Sec. III-B, Eq. 1-3: cosine similarity of the query embedding with every
                  chunk embedding, the two thresholds from the extreme scores, and the
                  bitwidth of every chunk by the comparisons of Alg. 1's prefill loop.
  append_tokens   Sec. III-A: the K/V rows of tokens generated during decoding are
                  kept in FP16 after the context; attention then runs over the
                  three context blocks followed by those rows.
  fold_appended   Sec. III-A: those rows become context (the FP16 list grows at
                  its end; a chunk they complete is an FP16 chunk).
  pack_* / unpack_*   the byte layout of the packed cache (an encoding this
                  build defines; the paper is silent on it).  V has a second form,
                  "token quads" (pack_quad_blocks), for grouped-query shapes.

Parity pins (tests/test_oracle_pins.py): all-FP16 equals textbook attention and
torch's scaled_dot_product_attention; invariance to the chunk permutation
(Sec. III-C, Eq. 4-5); |x - dequant(x)| <= scale/2; closed-form groups; a
scalar-loop brute force on tiny inputs; partial-softmax merge identity; pack
round trips; the KV-size figure of Sec. I; appended tokens equal textbook
attention over the concatenation and behave exactly like the FP16 remainder of a
longer context, and folding them in gives the cache of that longer context; the similarity scores equal scikit-learn's cosine_similarity,
and the thresholds a worked example, their limiting cases and their monotonicity
in alpha and beta.  No function here is unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

# Class index = position in the concatenation of Alg. 1's decode phase (INT2, INT4, FP16 there).  INT8,
# which the paper names as a further bitwidth (Sec. I), takes its place by precision: INT2, INT4, INT8, FP16.
CLASS_BITS = (2, 4, 8, 16)
NUM_CLASSES = len(CLASS_BITS)
FP16_CLASS = NUM_CLASSES - 1
TOKENS_PER_BLOCK = 64


def class_of_bits(bits: int) -> int:
    return {2: 0, 4: 1, 8: 2, 16: 3}[int(bits)]


# --------------------------------------------------------------------------- plan
@dataclass
class SeqPlan:
    perm: np.ndarray            # int32 [N]: reordered position j holds original chunk perm[j]
    class_chunks: Tuple[int, ...]        # per class
    class_tokens: Tuple[int, ...]        # per class; the FP16 count includes the unchunked tail
    tail: int


def plan_sequence(seq_len: int, chunk_size: int, bits: np.ndarray) -> SeqPlan:
    """Alg. 1 prefill loop for one sequence (stable partition by bitwidth)."""
    n = seq_len // chunk_size
    bits = np.asarray(bits)
    assert bits.shape == (n,)
    # a stable partition by class: INT2 chunks first, then INT4, INT8, FP16, each in original order
    cls = np.array([class_of_bits(x) for x in bits], dtype=np.int64)
    perm = np.argsort(cls, kind="stable").astype(np.int32)
    tail = seq_len - n * chunk_size          # Sec. III-A: remainder kept in FP16
    cc = tuple(int((cls == c).sum()) for c in range(NUM_CLASSES))
    ct = tuple(cc[c] * chunk_size + (tail if c == FP16_CLASS else 0) for c in range(NUM_CLASSES))
    return SeqPlan(perm, cc, ct, tail)


def class_token_index(seq_len: int, chunk_size: int, sp: SeqPlan) -> List[np.ndarray]:
    """For each class, the original token index of every token of that class, in cache order."""
    out = []
    pos = 0
    for c in range(NUM_CLASSES):
        chunks = sp.perm[pos:pos + sp.class_chunks[c]]
        pos += sp.class_chunks[c]
        idx = (chunks[:, None].astype(np.int64) * chunk_size + np.arange(chunk_size)[None, :]).reshape(-1)
        if c == FP16_CLASS and sp.tail:
            idx = np.concatenate([idx, np.arange(seq_len - sp.tail, seq_len, dtype=np.int64)])
        out.append(idx.astype(np.int64))
    return out


# ----------------------------------------------------------------------- quantize
def quantize_rows(x: np.ndarray, bits: int, group: int):
    """Per-token asymmetric min/max quantisation in groups along the last axis.

    x: fp16 [..., D].  Returns codes uint8 [..., D], scale fp16 [..., D/G], zero fp16 [..., D/G].
    Every step is one IEEE binary32 operation, round-to-nearest-even, unfused:
      mn, mx = min, max of the group (exact; zeros of either sign compare equal, so a zero
               minimum or maximum is taken as +0)
      r      = f32(mx) - f32(mn)
      scale  = f16(r / qmax)                       qmax = 2^bits - 1
      codes  = 0                                   if scale == 0
             = clamp(rint((f32(x) - f32(mn)) * (1 / f32(scale))), 0, qmax)   otherwise
    """
    assert x.dtype == np.float16 and bits in (2, 4, 8)
    d = x.shape[-1]
    assert d % group == 0
    qmax = np.float32((1 << bits) - 1)
    xg = x.reshape(x.shape[:-1] + (d // group, group))
    mn = xg.min(axis=-1)
    mx = xg.max(axis=-1)
    mn = np.where(mn == 0, np.float16(0.0), mn).astype(np.float16)
    mx = np.where(mx == 0, np.float16(0.0), mx).astype(np.float16)
    mn32 = mn.astype(np.float32)
    r = mx.astype(np.float32) - mn32
    scale = (r / qmax).astype(np.float16)
    sc32 = scale.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.float32(1.0) / sc32
    diff = xg.astype(np.float32) - mn32[..., None]
    with np.errstate(invalid="ignore", over="ignore"):
        t = np.rint(diff * inv[..., None])
    t = np.where(sc32[..., None] == 0, np.float32(0.0), t)
    codes = np.clip(t, np.float32(0.0), qmax).astype(np.uint8)
    return codes.reshape(x.shape), scale, mn


def dequantize(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray, group: int) -> np.ndarray:
    """x_hat = zero + code * scale in float64 (the definition of the encoding's value)."""
    d = codes.shape[-1]
    cg = codes.reshape(codes.shape[:-1] + (d // group, group)).astype(np.float64)
    xh = zero.astype(np.float64)[..., None] + cg * scale.astype(np.float64)[..., None]
    return xh.reshape(codes.shape)


# --------------------------------------------------------------------------- pack
def pack_row_words(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes uint8 [..., D] -> uint32 words [..., D*bits/32].

    Word k covers the n = 32/bits channels base = k*n ... base+n-1.  Channel
    base+2f sits at bits [f*bits, f*bits+bits) (low half-word = even channels),
    channel base+2f+1 at bits [16+f*bits, ...) (high half-word = odd channels).
    """
    n = 32 // bits
    d = codes.shape[-1]
    assert d % n == 0
    c = codes.reshape(codes.shape[:-1] + (d // n, n)).astype(np.uint32)
    w = np.zeros(c.shape[:-1], dtype=np.uint32)
    for f in range(n // 2):
        w |= c[..., 2 * f] << np.uint32(f * bits)
        w |= c[..., 2 * f + 1] << np.uint32(16 + f * bits)
    return w


def unpack_row_words(words: np.ndarray, bits: int) -> np.ndarray:
    n = 32 // bits
    mask = np.uint32((1 << bits) - 1)
    out = np.zeros(words.shape + (n,), dtype=np.uint8)
    for f in range(n // 2):
        out[..., 2 * f] = ((words >> np.uint32(f * bits)) & mask).astype(np.uint8)
        out[..., 2 * f + 1] = ((words >> np.uint32(16 + f * bits)) & mask).astype(np.uint8)
    return out.reshape(words.shape[:-1] + (words.shape[-1] * n,))


def block_bytes(cls: int, head_dim: int, group: int) -> int:
    bits = CLASS_BITS[cls]
    if bits == 16:
        return TOKENS_PER_BLOCK * head_dim * 2
    return TOKENS_PER_BLOCK * (head_dim * bits // 8 + 4 * head_dim // group)


def _pack_head_blocks(row_bytes: np.ndarray, meta_bytes) -> np.ndarray:
    """row_bytes uint8 [n, R] (R multiple of 16), meta_bytes uint8 [n, M] or None ->
    uint8 [nblk, block_bytes]: per 64-token block, 16-byte piece p of token i at
    (p*64 + i)*16, then the meta of token i at 64*R + i*M; missing tokens are zero."""
    n, rb = row_bytes.shape
    assert rb % 16 == 0, "head_dim must be a multiple of 64 (an INT2 row is a whole number of 16-byte pieces)"
    tb = TOKENS_PER_BLOCK
    nblk = (n + tb - 1) // tb
    pieces = rb // 16
    padded = np.zeros((nblk * tb, rb), dtype=np.uint8)
    padded[:n] = row_bytes
    codes = padded.reshape(nblk, tb, pieces, 16).transpose(0, 2, 1, 3).reshape(nblk, tb * rb)
    if meta_bytes is None:
        return np.ascontiguousarray(codes)
    mb = meta_bytes.shape[1]
    mp = np.zeros((nblk * tb, mb), dtype=np.uint8)
    mp[:n] = meta_bytes
    return np.concatenate([codes, mp.reshape(nblk, tb * mb)], axis=1)


def _unpack_head_blocks(buf: np.ndarray, n: int, rb: int, mb: int):
    tb = TOKENS_PER_BLOCK
    nblk = buf.shape[0]
    pieces = rb // 16
    codes = buf[:, :tb * rb].reshape(nblk, pieces, tb, 16).transpose(0, 2, 1, 3).reshape(nblk * tb, rb)[:n]
    meta = buf[:, tb * rb:].reshape(nblk * tb, mb)[:n] if mb else None
    return codes, meta


def pack_quad_blocks(vals: np.ndarray, bits: int, meta_bytes) -> np.ndarray:
    """The "token quads" form of a V block (used when 2 to 4 query heads share a kv head).

    vals: uint16 [n, D] codes (bits 2 or 4) or raw fp16 bit patterns (bits 16); D a multiple of 64.
    Same block size and piece addressing as _pack_head_blocks, but a 16-byte piece no longer holds
    one token: slot sl of piece p belongs to the token quad 4*(sl//4) .. +3 and to 16 channels.
    With n = 16/bits values per half-word, token i of the block, channel c:
        half  h = c // 64            lane of the quad  j = (c % 32) // 8
        e     = 8 * ((c % 64) // 32) + c % 8          (the j-th lane's e-th channel, 0..15)
        slot  sl = 4 * (i // 4) + j
        word  w = 2 * (e // n) + (i % 4) // 2          (of the 4 * pieces/2 words of half h)
        piece p = (pieces/2) * h + w // 4,  word of the piece = w % 4
        the value sits in the low (i even) or high (i odd) half-word at bit (e % n) * bits.
    So a word pairs two tokens of the quad for the same channels, and two consecutive words
    cover all four.  The meta bytes (scale, zero per token and group) follow as in the row form."""
    n, d = vals.shape
    assert d % 64 == 0 and bits in (2, 4, 8, 16)
    tb = TOKENS_PER_BLOCK
    nblk = (n + tb - 1) // tb
    per = 16 // bits
    rb = d * bits // 8
    pieces = rb // 16
    hw = np.zeros((nblk, pieces, tb, 4, 2), dtype=np.uint16)      # [block][piece][slot][word][half-word]
    tok = np.arange(n)[:, None] + np.zeros((1, d), dtype=np.int64)
    c = np.zeros((n, 1), dtype=np.int64) + np.arange(d)[None, :]
    i = tok % tb
    h = c // 64
    j = (c % 32) // 8
    e = 8 * ((c % 64) // 32) + c % 8
    sl = 4 * (i // 4) + j
    w = 2 * (e // per) + (i % 4) // 2
    pc = (pieces // (d // 64)) * h + w // 4
    shifted = (vals.astype(np.uint32) << ((e % per) * bits).astype(np.uint32)).astype(np.uint16)
    np.add.at(hw, (tok // tb, pc, sl, w % 4, i % 2), shifted)      # disjoint bit fields: add = or
    codes = hw.astype("<u2").view(np.uint8).reshape(nblk, tb * rb)
    if meta_bytes is None:
        return np.ascontiguousarray(codes)
    mb = meta_bytes.shape[1]
    mp = np.zeros((nblk * tb, mb), dtype=np.uint8)
    mp[:n] = meta_bytes
    return np.concatenate([codes, mp.reshape(nblk, tb * mb)], axis=1)


def unpack_quad_blocks(buf: np.ndarray, n: int, d: int, bits: int, mb: int):
    """Inverse of pack_quad_blocks: (uint16 [n, d] values, meta bytes or None)."""
    tb = TOKENS_PER_BLOCK
    nblk = buf.shape[0]
    per = 16 // bits
    rb = d * bits // 8
    pieces = rb // 16
    hw = np.ascontiguousarray(buf[:, :tb * rb]).view("<u2").reshape(nblk, pieces, tb, 4, 2)
    out = np.zeros((n, d), dtype=np.uint16)
    mask = (1 << bits) - 1
    for t in range(n):
        blk, i = divmod(t, tb)
        for c in range(d):
            e = 8 * ((c % 64) // 32) + c % 8
            w = 2 * (e // per) + (i % 4) // 2
            piece = (pieces // (d // 64)) * (c // 64) + w // 4
            x = int(hw[blk, piece, 4 * (i // 4) + (c % 32) // 8, w % 4, i % 2])
            out[t, c] = (x >> ((e % per) * bits)) & mask
    meta = buf[:, tb * rb:].reshape(nblk * tb, mb)[:n] if mb else None
    return out, meta


@dataclass
class ClassCache:
    """Logical content of one class for one sequence (all kv heads)."""
    bits: int
    n_tokens: int
    k_codes: np.ndarray = None   # uint8 [Hkv, n, D]   (quantised classes)
    k_scale: np.ndarray = None   # fp16  [Hkv, n, D/G]
    k_zero: np.ndarray = None
    v_codes: np.ndarray = None
    v_scale: np.ndarray = None
    v_zero: np.ndarray = None
    k_raw: np.ndarray = None     # fp16 [Hkv, n, D]    (FP16 class)
    v_raw: np.ndarray = None


@dataclass
class OracleCache:
    head_dim: int
    group: int
    chunk_size: int
    num_kv_heads: int
    plans: List[SeqPlan]
    seqs: List[List[ClassCache]]         # [B][NUM_CLASSES]
    app_k: List[np.ndarray] = None       # [B] fp16 [Hkv, n_app, D]: rows appended during decoding
    app_v: List[np.ndarray] = None
    seq_lens: List[int] = None           # [B] context tokens T_b
    bits: List[np.ndarray] = None        # [B] uint8 [N_b]: the bitwidth of every chunk


def reorder_quantize(k_seqs: Sequence[np.ndarray], v_seqs: Sequence[np.ndarray],
                     bits_seqs: Sequence[np.ndarray], chunk_size: int, group: int) -> OracleCache:
    """Alg. 1 prefill phase: gather each class's chunks (reorder), then quantise the INT2/INT4 lists.

    k_seqs[b], v_seqs[b]: fp16 [Hkv, T_b, D].
    """
    plans, seqs = [], []
    hkv, _, d = k_seqs[0].shape
    for k, v, bits in zip(k_seqs, v_seqs, bits_seqs):
        t = k.shape[1]
        sp = plan_sequence(t, chunk_size, bits)
        idx = class_token_index(t, chunk_size, sp)
        ccs = []
        for c in range(NUM_CLASSES):
            kc, vc = k[:, idx[c], :], v[:, idx[c], :]          # the reordered, contiguous class
            cc = ClassCache(CLASS_BITS[c], len(idx[c]))
            if c == FP16_CLASS:
                cc.k_raw, cc.v_raw = np.ascontiguousarray(kc), np.ascontiguousarray(vc)
            else:
                cc.k_codes, cc.k_scale, cc.k_zero = quantize_rows(kc, CLASS_BITS[c], group)
                cc.v_codes, cc.v_scale, cc.v_zero = quantize_rows(vc, CLASS_BITS[c], group)
            ccs.append(cc)
        plans.append(sp)
        seqs.append(ccs)
    empty = [np.zeros((hkv, 0, d), dtype=np.float16) for _ in plans]
    return OracleCache(d, group, chunk_size, hkv, plans, seqs, empty, [e.copy() for e in empty],
                       [int(k.shape[1]) for k in k_seqs], [np.asarray(x, dtype=np.uint8).copy() for x in bits_seqs])


def gather_pages(pages: np.ndarray, table_row: Sequence[int], seq_len: int) -> np.ndarray:
    """A sequence's K (or V) from a paged cache: pages fp16 [num_pages, Hkv, page_size, D]; token t of the
    sequence is slot t % page_size of page table_row[t // page_size].  Returns fp16 [Hkv, seq_len, D], the
    input of reorder_quantize (Alg. 1 starts from the K, V of the whole context)."""
    page_size = pages.shape[2]
    out = np.empty((pages.shape[1], seq_len, pages.shape[3]), dtype=pages.dtype)
    for t in range(seq_len):
        out[:, t, :] = pages[table_row[t // page_size], :, t % page_size, :]
    return out


def append_tokens(cache: OracleCache, k_new: np.ndarray, v_new: np.ndarray, active: Sequence[bool] = None) -> None:
    """Sec. III-A: one generated token per sequence joins the cache in FP16, behind everything else.

    k_new, v_new: fp16 [B, Hkv, D].  active: which sequences generated a token in this step (all by default);
    the rows of the others are ignored, so sequences may stop generating at different steps.
    """
    for b in range(len(cache.seqs)):
        if active is not None and not active[b]:
            continue
        cache.app_k[b] = np.concatenate([cache.app_k[b], k_new[b][:, None, :].astype(np.float16)], axis=1)
        cache.app_v[b] = np.concatenate([cache.app_v[b], v_new[b][:, None, :].astype(np.float16)], axis=1)


def fold_appended(cache: OracleCache) -> None:
    """Sec. III-A: the rows appended during decoding become context.  T_b grows by their number; they stay FP16
    and stay where they are in the order of the tokens, behind the remainder of the context, so the FP16 list of
    Alg. 1 simply grows at its end; a chunk that they complete is an FP16 chunk (bitwidth 16).  Afterwards nothing
    is appended any more, and the cache is the one reorder_quantize builds from the longer context."""
    for b, ccs in enumerate(cache.seqs):
        n = cache.app_k[b].shape[1]
        if n == 0:
            continue
        fp = ccs[FP16_CLASS]
        fp.k_raw = np.concatenate([fp.k_raw, cache.app_k[b]], axis=1)
        fp.v_raw = np.concatenate([fp.v_raw, cache.app_v[b]], axis=1)
        fp.n_tokens += n
        t = cache.seq_lens[b] + n
        completed = t // cache.chunk_size - cache.bits[b].size
        cache.bits[b] = np.concatenate([cache.bits[b], np.full(completed, 16, dtype=np.uint8)])
        cache.seq_lens[b] = t
        cache.plans[b] = plan_sequence(t, cache.chunk_size, cache.bits[b])
        cache.app_k[b] = cache.app_k[b][:, :0, :]
        cache.app_v[b] = cache.app_v[b][:, :0, :]


def pack_append_buffer(cache: OracleCache, which: str, capacity: int, v_quads: bool = False) -> np.ndarray:
    """Byte image of the append buffer: per (sequence, kv head) ceil(capacity/64) FP16 blocks in the
    block layout of the FP16 class (V in token quads if v_quads); rows not appended yet are zero bytes."""
    nblk = (capacity + TOKENS_PER_BLOCK - 1) // TOKENS_PER_BLOCK
    rb = 2 * cache.head_dim
    parts = []
    for b in range(len(cache.seqs)):
        src = cache.app_k[b] if which == "k" else cache.app_v[b]
        for h in range(cache.num_kv_heads):
            rows = np.zeros((nblk * TOKENS_PER_BLOCK, rb), dtype=np.uint8)
            n = src.shape[1]
            rows[:n] = np.ascontiguousarray(src[h]).view(np.uint8).reshape(n, rb)
            if v_quads and which == "v":
                parts.append(pack_quad_blocks(np.ascontiguousarray(rows).view("<u2"), 16, None).reshape(-1))
            else:
                parts.append(_pack_head_blocks(rows, None).reshape(-1))
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.uint8)


def _rows_and_meta(cc: ClassCache, which: str, h: int):
    if cc.bits == 16:
        raw = cc.k_raw if which == "k" else cc.v_raw
        return np.ascontiguousarray(raw[h]).view(np.uint8).reshape(cc.n_tokens, -1), None
    codes = (cc.k_codes if which == "k" else cc.v_codes)[h]
    scale = (cc.k_scale if which == "k" else cc.v_scale)[h]
    zero = (cc.k_zero if which == "k" else cc.v_zero)[h]
    words = pack_row_words(codes, cc.bits).astype("<u4")
    rows = words.view(np.uint8).reshape(cc.n_tokens, -1)
    meta = np.stack([scale.astype("<f2"), zero.astype("<f2")], axis=-1)      # [n, D/G, 2]
    return rows, np.ascontiguousarray(meta).view(np.uint8).reshape(cc.n_tokens, -1)


def _values_and_meta(cc: ClassCache, h: int):
    """V of head h as uint16 values per channel (codes, or fp16 bit patterns) and the meta bytes."""
    if cc.bits == 16:
        return np.ascontiguousarray(cc.v_raw[h]).view("<u2").reshape(cc.n_tokens, -1), None
    meta = np.stack([cc.v_scale[h].astype("<f2"), cc.v_zero[h].astype("<f2")], axis=-1)
    return cc.v_codes[h].astype(np.uint16), np.ascontiguousarray(meta).view(np.uint8).reshape(cc.n_tokens, -1)


def pack_class_buffer(cache: OracleCache, cls: int, which: str, v_quads: bool = False,
                      reserve: Sequence[int] = None) -> np.ndarray:
    """Bytes of the K (or V) device buffer of one class: blocks ordered by (sequence, kv head, block).
    v_quads: V is stored in the token-quad form (pack_quad_blocks); K is not affected.
    reserve: the FP16 runs of sequence b are laid out with room for reserve[b] more tokens (a cache that appended
    rows are folded into later): every (sequence, kv head) run of the FP16 class is followed by zero blocks up to
    ceil((n + reserve[b]) / 64) blocks."""
    parts = []
    bb = block_bytes(cls, cache.head_dim, cache.group)
    for b, ccs in enumerate(cache.seqs):
        cc = ccs[cls]
        room = reserve[b] if (reserve is not None and cls == FP16_CLASS) else 0
        nblk = (cc.n_tokens + TOKENS_PER_BLOCK - 1) // TOKENS_PER_BLOCK
        spare = (cc.n_tokens + room + TOKENS_PER_BLOCK - 1) // TOKENS_PER_BLOCK - nblk
        for h in range(cache.num_kv_heads):
            if cc.n_tokens:
                if v_quads and which == "v":
                    vals, meta = _values_and_meta(cc, h)
                    parts.append(pack_quad_blocks(vals, cc.bits, meta).reshape(-1))
                else:
                    rows, meta = _rows_and_meta(cc, which, h)
                    parts.append(_pack_head_blocks(rows, meta).reshape(-1))
            if spare:
                parts.append(np.zeros(spare * bb, dtype=np.uint8))
    if not parts:
        return np.zeros(0, dtype=np.uint8)
    return np.concatenate(parts)


def unpack_class_buffer(buf: np.ndarray, cache_like: OracleCache, cls: int):
    """Inverse of pack_class_buffer: per sequence, per head (codes-or-raw, scale, zero)."""
    d, g = cache_like.head_dim, cache_like.group
    bits = CLASS_BITS[cls]
    rb = d * 2 if bits == 16 else d * bits // 8
    mb = 0 if bits == 16 else 4 * d // g
    bb = block_bytes(cls, d, g)
    out, pos = [], 0
    for ccs in cache_like.seqs:
        n = ccs[cls].n_tokens
        nblk = (n + TOKENS_PER_BLOCK - 1) // TOKENS_PER_BLOCK
        heads = []
        for _ in range(cache_like.num_kv_heads if n else 0):
            blk = buf[pos:pos + nblk * bb].reshape(nblk, bb)
            pos += nblk * bb
            rows, meta = _unpack_head_blocks(blk, n, rb, mb)
            if bits == 16:
                heads.append((np.ascontiguousarray(rows).view("<f2").reshape(n, d), None, None))
            else:
                codes = unpack_row_words(np.ascontiguousarray(rows).view("<u4").reshape(n, -1), bits)
                m = np.ascontiguousarray(meta).view("<f2").reshape(n, d // g, 2)
                heads.append((codes, m[..., 0], m[..., 1]))
        out.append(heads)
    assert pos == buf.size
    return out


def dequantized_kv(cache: OracleCache, b: int, h: int) -> Tuple[np.ndarray, np.ndarray]:
    """float64 [n_total, D] K-hat and V-hat of (b, kv head h) in cache order INT2 | INT4 | INT8 | FP16 | appended."""
    ks, vs = [], []
    for cc in cache.seqs[b]:
        if cc.bits == 16:
            ks.append(cc.k_raw[h].astype(np.float64))
            vs.append(cc.v_raw[h].astype(np.float64))
        else:
            ks.append(dequantize(cc.k_codes[h], cc.k_scale[h], cc.k_zero[h], cache.group))
            vs.append(dequantize(cc.v_codes[h], cc.v_scale[h], cc.v_zero[h], cache.group))
    if cache.app_k is not None:
        ks.append(cache.app_k[b][h].astype(np.float64))
        vs.append(cache.app_v[b][h].astype(np.float64))
    return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)


# ---------------------------------------------------------------------- attention
def attention_head(q: np.ndarray, kh: np.ndarray, vh: np.ndarray, sm_scale: float):
    """softmax(sm_scale * q K^T) V for one query vector, float64.  Returns (out [D], lse)."""
    if kh.shape[0] == 0:
        return np.zeros(vh.shape[1], dtype=np.float64), -np.inf
    s = sm_scale * (kh @ q.astype(np.float64))
    m = s.max()
    e = np.exp(s - m)
    l = e.sum()
    return (e / l) @ vh, m + np.log(l)


def decode_attention(q: np.ndarray, cache: OracleCache, sm_scale: float = None,
                     heads: Sequence[Tuple[int, int]] = None):
    """Alg. 1 decode phase for every (sequence, query head), or only those in `heads`.

    q: fp16 [B, Hq, D].  Returns out float64 [B, Hq, D] and lse float64 [B, Hq]
    (entries not in `heads` are NaN).
    """
    bsz, hq, d = q.shape
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    rep = hq // cache.num_kv_heads
    out = np.full((bsz, hq, d), np.nan)
    lse = np.full((bsz, hq), np.nan)
    todo = heads if heads is not None else [(b, h) for b in range(bsz) for h in range(hq)]
    memo: Dict[Tuple[int, int], Tuple[np.ndarray, np.ndarray]] = {}
    for b, h in todo:
        key = (b, h // rep)
        if key not in memo:
            memo.clear()
            memo[key] = dequantized_kv(cache, b, h // rep)
        kh, vh = memo[key]
        out[b, h], lse[b, h] = attention_head(q[b, h], kh, vh, sm_scale)
    return out, lse


def merge_partials(ms: Sequence[float], ls: Sequence[float], os_: Sequence[np.ndarray]):
    """Exact merge of partial softmax states (m_i, l_i, o_i): o_i = sum_t e^{s_t - m_i} v_t."""
    ms = np.asarray(ms, dtype=np.float64)
    ls = np.asarray(ls, dtype=np.float64)
    if len(ms) == 0 or not np.any(ls > 0):
        return None, -np.inf
    m = ms[ls > 0].max()
    w = np.where(ls > 0, np.exp(np.where(ls > 0, ms, m) - m), 0.0)
    big_l = float((w * ls).sum())
    o = sum(wi * np.asarray(oi, dtype=np.float64) for wi, oi in zip(w, os_))
    return o / big_l, m + np.log(big_l)


# ---------------------------------------------------------------------- footprint
def kv_bytes_fp16(layers: int, heads: int, head_dim: int, tokens: int) -> int:
    """Bytes of an un-quantised fp16 KV cache (K and V)."""
    return layers * heads * head_dim * tokens * 2 * 2


def packed_bytes(class_tokens: Sequence[int], num_kv_heads: int, head_dim: int, group: int) -> int:
    """Algorithmic bytes (K + V) of the packed cache of one sequence: codes + fp16 scale/zero per group."""
    per = [head_dim * b // 8 + (4 * head_dim // group if b < 16 else 0) for b in CLASS_BITS]
    return 2 * num_kv_heads * sum(n * p for n, p in zip(class_tokens, per))


# ---------------------------------------------------------------------- chunk-level quantization search
def similarity_scores(query_emb: np.ndarray, chunk_emb: np.ndarray) -> np.ndarray:
    """Sec. III-B, Eq. 1: cosine similarity of one query embedding [E] with every chunk embedding [N, E].

    Evaluated in float64 and rounded once to float32, the precision in which the thresholds are
    compared.  A zero vector has no direction: its score is taken as 0.
    """
    q = query_emb.astype(np.float64)
    c = chunk_emb.astype(np.float64)
    dots = c @ q
    denom = np.sqrt(q @ q) * np.sqrt(np.einsum("ne,ne->n", c, c))
    s = np.divide(dots, denom, out=np.zeros_like(dots), where=denom > 0)
    return s.astype(np.float32)


def thresholds(scores: np.ndarray, alpha: float, beta: float):
    """Sec. III-B, Eq. 2-3 in float32, one rounding per operation:
    T_low = s_min + (s_max - s_min) * alpha,  T_high = s_max - (s_max - s_min) * beta."""
    smin, smax = np.float32(scores.min()), np.float32(scores.max())
    d = np.float32(smax - smin)
    t_low = np.float32(smin + np.float32(d * np.float32(alpha)))
    t_high = np.float32(smax - np.float32(d * np.float32(beta)))
    return t_low, t_high


def chunk_bitwidths(query_emb: np.ndarray, chunk_emb: np.ndarray, alpha: float, beta: float):
    """Chunk-level quantization search for one sequence (Sec. III-B) with the comparison order of
    Alg. 1's prefill loop: s < T_low -> INT2, else s > T_high -> FP16, else INT4.

    Returns (bits uint8 [N] with values 2 / 4 / 16, scores float32 [N]).
    """
    n = chunk_emb.shape[0]
    if n == 0:
        return np.zeros(0, dtype=np.uint8), np.zeros(0, dtype=np.float32)
    s = similarity_scores(query_emb, chunk_emb)
    t_low, t_high = thresholds(s, alpha, beta)
    bits = np.full(n, 4, dtype=np.uint8)
    for i in range(n):
        if s[i] < t_low:
            bits[i] = 2
        elif s[i] > t_high:
            bits[i] = 16
    return bits, s
