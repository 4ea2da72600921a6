"""Host logic of libcocktail.so (no GPU): symbols, argument validation, planner vs oracle, work split."""
import ctypes as C
import os
import re
import struct

import numpy as np
import pytest

import workloads
from oracle import cocktail_oracle as O
import paper_2503_23294_amd as ck
from paper_2503_23294_amd import _lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "cocktail.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(cocktail_[a-z_]+)\s*\(", hdr))
    assert declared == set(_lib.EXPORTS), declared ^ set(_lib.EXPORTS)
    handle = _lib.lib()
    for name in declared:
        assert getattr(handle, name) is not None
    assert handle.cocktail_version() >= 1


def _plan(w, workers):
    sh = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = workloads.chunk_bits(w)
    flat = np.concatenate(bits) if bits else np.zeros(0, np.uint8)
    return ck.cocktail_plan(sh, w.seq_lens, flat, workers), bits


# field offsets of the internal plan header (csrc/plan.h), little-endian
_HDR = struct.Struct("<II6i i3i ii qq 3q3q 3i3i qqq 11i i 4i")


def _parse(blob):
    f = _HDR.unpack_from(blob.tobytes(), 0)
    names = ["magic", "version", "batch", "hq", "hkv", "d", "chunk", "group", "rep", "workers", "segments",
             "partials", "gblocks", "pad0", "total_chunks", "total_tokens"]
    h = dict(zip(names, f[:16]))
    h["class_blocks"], h["class_bytes"] = f[16:19], f[19:22]
    h["block_bytes"], h["row_bytes"] = f[22:25], f[25:28]
    h["workspace_bytes"], h["plan_bytes"], h["packed_bytes"] = f[28:31]
    offs = f[31:42]
    keys = ["seq_len", "cum_tokens", "chunk_off", "perm", "class_tokens", "class_chunk0", "blk_base", "nblk",
            "segments", "bh_pid", "worker_rec"]
    h["off"] = dict(zip(keys, offs))
    h["items"] = f[42]
    return h


def _arr(blob, off, dtype, n):
    return np.frombuffer(blob.tobytes(), dtype=dtype, count=n, offset=off)


@pytest.mark.parametrize("cfg,workers", [(1, 64), (1, 2048), (3, 512), (4, 2048), (5, 512), (5, 7)])
def test_planner_matches_oracle_and_splits_work_exactly_once(cfg, workers):
    w = workloads.config(cfg)
    plan, bits = _plan(w, workers)
    pos = 0
    packed = 0
    for b, t in enumerate(w.seq_lens):
        sp = O.plan_sequence(t, w.chunk_size, bits[b])
        n = t // w.chunk_size
        assert plan.perm[pos:pos + n].tolist() == sp.perm.tolist()
        assert tuple(plan.class_tokens[b]) == sp.class_tokens
        packed += O.packed_bytes(sp.class_tokens, w.num_kv_heads, w.head_dim, w.group_size)
        pos += n
    assert plan.sizes.packed_bytes == packed
    for c in range(3):
        blocks = sum(((int(plan.class_tokens[b, c]) + 63) // 64) * w.num_kv_heads for b in range(w.batch))
        assert plan.sizes.class_blocks[c] == blocks
        assert plan.sizes.class_bytes[c] == blocks * O.block_bytes(c, w.head_dim, w.group_size)

    h = _parse(plan.blob)
    assert h["plan_bytes"] == plan.blob.size and h["workers"] == workers
    S, P, Q = h["segments"], workers, h["items"]
    segs = _arr(plan.blob, h["off"]["segments"], np.int32, 8 * S).reshape(S, 8)
    BH = w.batch * w.num_kv_heads
    bh_pid = _arr(plan.blob, h["off"]["bh_pid"], np.int32, BH * 12).reshape(BH, 3, 2, 2)
    recs = _arr(plan.blob, h["off"]["worker_rec"], np.int32, 16 * (P + Q)).reshape(P + Q, 16)
    assert h["gblocks"] == sum(plan.sizes.class_blocks)
    # segments tile the class buffers: every physical block of every (class, b, h) exactly once
    phys = [np.zeros(int(plan.sizes.class_blocks[c]), dtype=np.int32) for c in range(3)]
    g = 0
    for b_, h_, cls, ntok, blk0, nblk, gblk0, bh in segs:
        assert gblk0 == g and bh == b_ * w.num_kv_heads + h_ and nblk > 0 and ntok > (nblk - 1) * 64
        phys[cls][blk0:blk0 + nblk] += 1
        g += nblk
    assert all((x == 1).all() for x in phys)
    # walk every work item the way the kernel does; every block is visited exactly once
    seen = np.zeros(h["gblocks"], dtype=np.int32)
    pid_owner = {}
    cost = []
    for it in range(P + Q):
        g, g1, s, pid = recs[it, :4]
        if g < g1:
            assert recs[it, 4:12].tolist() == segs[s].tolist()
        cur = None
        bytes_ = 0
        while g < g1:
            b_, h_, cls, ntok, blk0, nblk, gblk0, bh = segs[s]
            assert gblk0 <= g < gblk0 + nblk
            if (cls, bh) != cur:
                if cur is not None:
                    pid += 1
                cur = (cls, bh)
                assert pid not in pid_owner
                pid_owner[pid] = (cls, bh, 0 if it < P else 1)
            je = min(gblk0 + nblk, g1)
            seen[g:je] += 1
            bytes_ += (je - g) * 2 * h["block_bytes"][cls]
            g = je
            s += 1
        cost.append(bytes_)
    assert (seen == 1).all()
    assert sorted(pid_owner) == list(range(h["partials"])) and h["partials"] == plan.sizes.num_partials
    covered = 0
    for bh in range(BH):
        for c in range(3):
            for part in range(2):
                lo, hi = bh_pid[bh, c, part]
                assert all(pid_owner[p] == (c, bh, part) for p in range(lo, hi))
                covered += hi - lo
    assert covered == h["partials"]
    # the static ranges carry most of the bytes; dynamic items are small
    static, dyn = cost[:P], cost[P:]
    total = sum(cost)
    if Q:
        assert 0.05 * total <= sum(dyn) <= 0.35 * total
        assert max(dyn) <= 64 * 1024
    assert plan.sizes.workspace_bytes == max(h["partials"], 1) * h["rep"] * (w.head_dim + 2) * 4


def test_plan_handles_empty_sequences_and_tail_only():
    sh = ck.make_shape(3, 2, 2, 128, 16, 32)
    plan = ck.cocktail_plan(sh, [0, 5, 16], [4], 8)
    assert plan.class_tokens.tolist() == [[0, 0, 0], [0, 0, 5], [0, 16, 0]]
    assert list(plan.sizes.class_blocks) == [0, 2, 2] and plan.sizes.num_partials >= 4


@pytest.mark.parametrize("kwargs,code", [
    (dict(hq=3, hkv=2), _lib.EINVAL), (dict(d=96), _lib.EINVAL), (dict(g=48), _lib.EINVAL),
    (dict(d=64, g=128), _lib.EINVAL), (dict(chunk=0), _lib.EINVAL), (dict(workers=0), _lib.EINVAL),
    (dict(bits=[2, 3]), _lib.EINVAL), (dict(lens=[-1]), _lib.EINVAL),
])
def test_plan_rejects_bad_arguments(kwargs, code):
    sh = ck.make_shape(1, kwargs.get("hq", 2), kwargs.get("hkv", 2), kwargs.get("d", 128), kwargs.get("chunk", 8),
                       kwargs.get("g", 32))
    lens = np.asarray(kwargs.get("lens", [16]), dtype=np.int32)
    bits = np.asarray(kwargs.get("bits", [2, 4]), dtype=np.uint8)
    sizes = _lib.Sizes()
    rc = _lib.lib().cocktail_plan(C.byref(sh), lens.ctypes.data_as(C.POINTER(C.c_int32)),
                                  bits.ctypes.data_as(C.POINTER(C.c_uint8)), kwargs.get("workers", 4),
                                  C.byref(sizes), None, 0, None, None)
    assert rc == code
    assert _lib.lib().cocktail_last_error() != b""


def test_plan_capacity_and_null_checks():
    sh = ck.make_shape(1, 2, 2, 128, 8, 32)
    lens = np.array([16], dtype=np.int32)
    bits = np.array([2, 4], dtype=np.uint8)
    sizes = _lib.Sizes()
    L = _lib.lib()
    lp, bp = lens.ctypes.data_as(C.POINTER(C.c_int32)), bits.ctypes.data_as(C.POINTER(C.c_uint8))
    assert L.cocktail_plan(C.byref(sh), lp, bp, 4, C.byref(sizes), None, 0, None, None) == _lib.OK
    small = np.zeros(16, dtype=np.uint8)
    assert L.cocktail_plan(C.byref(sh), lp, bp, 4, C.byref(sizes), small.ctypes.data, 16, None, None) == _lib.ENOSPACE
    assert L.cocktail_plan(C.byref(sh), None, bp, 4, C.byref(sizes), None, 0, None, None) == _lib.EINVAL
    assert L.cocktail_plan(C.byref(sh), lp, None, 4, C.byref(sizes), None, 0, None, None) == _lib.EINVAL
    assert L.cocktail_plan(None, lp, bp, 4, C.byref(sizes), None, 0, None, None) == _lib.EINVAL


def test_gpu_entry_points_validate_on_host_before_launching():
    """Bad arguments are rejected before any HIP call, so this runs without a GPU."""
    sh = ck.make_shape(1, 2, 2, 128, 8, 32)
    plan = ck.cocktail_plan(sh, [16], [2, 4], 4)
    L = _lib.lib()
    cache = _lib.Cache()
    assert L.cocktail_reorder_quantize(C.byref(sh), 16, 16, 0, 0, 0, 128, None, None) == _lib.EINVAL
    assert L.cocktail_reorder_quantize(C.byref(sh), 16, 16, 0, 0, 0, 128, C.byref(cache), None) == _lib.EINVAL
    cache.plan_host = plan.blob.ctypes.data
    cache.plan_dev = 4096
    assert L.cocktail_reorder_quantize(C.byref(sh), 8, 16, 0, 0, 0, 128, C.byref(cache), None) == _lib.EALIGN
    assert L.cocktail_reorder_quantize(C.byref(sh), 16, 16, 7, 0, 0, 128, C.byref(cache), None) == _lib.EINVAL
    assert L.cocktail_reorder_quantize(C.byref(sh), 16, 16, 0, 0, 0, 100, C.byref(cache), None) == _lib.EINVAL
    assert L.cocktail_reorder_quantize(C.byref(sh), 16, 16, 0, 0, 0, 128, C.byref(cache), None) == _lib.EINVAL  # NULL class buffers
    other = ck.make_shape(1, 2, 2, 128, 16, 32)
    assert L.cocktail_reorder_quantize(C.byref(other), 16, 16, 0, 0, 0, 128, C.byref(cache), None) == _lib.EINVAL
    assert b"different shape" in L.cocktail_last_error()
    assert L.cocktail_decode_attention(C.byref(sh), None, C.byref(cache), 0.0, 16, None, 16, 0, None) == _lib.EINVAL
    assert L.cocktail_decode_attention(C.byref(sh), 16, C.byref(cache), 0.0, 16, None, 16, 0, None) == _lib.ENOSPACE
    assert L.cocktail_decode_attention(C.byref(sh), 16, C.byref(cache), 0.0, 24, None, 16, 1 << 20, None) == _lib.EALIGN
    sh64 = ck.make_shape(1, 2, 2, 64, 8, 32)
    p64 = ck.cocktail_plan(sh64, [16], [2, 4], 4)
    cache.plan_host = p64.blob.ctypes.data
    assert L.cocktail_decode_attention(C.byref(sh64), 16, C.byref(cache), 0.0, 16, None, 16, 1 << 20, None) == _lib.EUNSUPPORTED
    sh16 = ck.make_shape(1, 16, 1, 128, 8, 32)
    p16 = ck.cocktail_plan(sh16, [16], [2, 4], 4)
    cache.plan_host = p16.blob.ctypes.data
    assert L.cocktail_decode_attention(C.byref(sh16), 16, C.byref(cache), 0.0, 16, None, 16, 1 << 20, None) == _lib.EUNSUPPORTED
    n = C.c_size_t(0)
    assert L.cocktail_stream_read_probe(None, 1 << 30, 16, C.byref(n), None) == _lib.EINVAL
    assert L.cocktail_stream_read_probe(8, 1 << 30, 16, C.byref(n), None) == _lib.EALIGN
    assert L.cocktail_stream_read_probe(16, 1 << 20, 16, C.byref(n), None) == _lib.EINVAL
