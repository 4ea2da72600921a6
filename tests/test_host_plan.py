"""Host logic of libcocktail.so (no GPU): symbols, argument validation, planner vs oracle, work split."""
import ctypes as C
import os
import re

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
    declared = set(re.findall(r"\b(cocktail_[a-z0-9_]+)\s*\(", hdr))
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


def _parse(plan):
    """The fields of the plan's internal header that these tests look at, read by name through the library's
    accessor, so that a change of the header layout cannot be misread here."""
    f = lambda name, i=0: ck.cocktail_plan_field(plan, name, i)
    h = {"rep": f("rep"), "workers": f("num_workers"), "segments": f("num_segments"), "partials": f("num_partials"),
         "gblocks": f("total_gblocks"), "v_layout": f("v_layout"), "plan_bytes": f("plan_bytes"),
         "work_heads": f("work_heads"), "work_rep": f("work_rep"),
         "groups": f("num_groups"), "pool_segs": f("num_pool_segs"), "ws_status_off": f("ws_status_off"),
         "block_bytes": [f("block_bytes", c) for c in range(_lib.NUM_CLASSES)]}
    h["off"] = {k: f("off_" + k) for k in ("segments", "worker_rec", "group_rec", "pool_seg", "counters", "bh_off")}
    assert f("sizeof_segment") == 32 and f("sizeof_worker_rec") == 64 and f("sizeof_group_rec") == 32
    assert f("sizeof_pool_seg") == 32
    return h


def _consts(plan):
    return ([ck.cocktail_plan_field(plan, "iter_units", c) for c in range(_lib.NUM_CLASSES)],
            ck.cocktail_plan_field(plan, "counter_stride_bytes") // 4, ck.cocktail_plan_field(plan, "partial_header_floats"))


def _arr(blob, off, dtype, n):
    return np.frombuffer(blob.tobytes(), dtype=dtype, count=n, offset=off)


def _check_work_split(plan, w, workers, seed=0):
    """Replays the decode kernel's walk over the plan (own ranges, then pool tickets in a random
    hand-out order) and checks that every unit is read exactly once and every partial id is sound."""
    h = _parse(plan)
    ITER_UNITS, COUNTER_STRIDE, header_floats = _consts(plan)
    # the requested number of workers is an upper bound: never more workers than units of work (multiples of 64)
    share = h["work_heads"] // w.num_kv_heads
    nc = _lib.NUM_CLASSES
    f = ck.cocktail_plan_field
    # blocks per head that hold tokens, blocks per head the run is laid out with (room to grow), first block per sequence
    used_blk = _arr(plan.blob, f(plan, "off_nblk"), np.int32, nc * w.batch).reshape(w.batch, nc)
    run_blk = _arr(plan.blob, f(plan, "off_run_blocks"), np.int32, nc * w.batch).reshape(w.batch, nc)
    base_blk = _arr(plan.blob, f(plan, "off_blk_base"), np.int32, nc * (w.batch + 1)).reshape(w.batch + 1, nc)
    work_blocks = int(used_blk.sum()) * w.num_kv_heads
    units = work_blocks * share * (1 if w.head_dim == 64 else 2)
    assert h["plan_bytes"] == plan.blob.size
    assert h["workers"] == plan.sizes.num_workers == min(workers, max((units + 63) // 64 * 64, 64))
    workers = h["workers"]
    S, P, NG, NPS = h["segments"], workers, h["groups"], h["pool_segs"]
    segs = _arr(plan.blob, h["off"]["segments"], np.int32, 8 * S).reshape(S, 8)
    BH = w.batch * h["work_heads"]
    bh_off = _arr(plan.blob, h["off"]["bh_off"], np.int32, BH + 1)
    recs = _arr(plan.blob, h["off"]["worker_rec"], np.int32, 16 * P).reshape(P, 16)
    groups = _arr(plan.blob, h["off"]["group_rec"], np.int32, 8 * NG).reshape(NG, 8)
    psegs = _arr(plan.blob, h["off"]["pool_seg"], np.int32, 8 * NPS).reshape(NPS, 8)
    counters = _arr(plan.blob, h["off"]["counters"], np.uint32, COUNTER_STRIDE * NG)
    assert (counters == 0).all() and h["off"]["counters"] % 128 == 0
    share = h["work_heads"] // w.num_kv_heads              # work heads that walk the blocks of one kv head
    assert h["gblocks"] == work_blocks * share
    # segments tile the class buffers: every physical block of every (class, b, h) exactly once per work head
    phys = [np.zeros(int(plan.sizes.class_blocks[c]), dtype=np.int32) for c in range(_lib.NUM_CLASSES)]
    g = 0
    for b_, h_, cls, ntok, blk0, nblk, gblk0, spid in segs:
        assert gblk0 == g and nblk > 0 and (nblk - 1) * 64 < ntok
        phys[cls][blk0:blk0 + nblk] += 1
        g += nblk
    for c in range(nc):
        want = np.zeros_like(phys[c])
        for b_ in range(w.batch):
            for h_ in range(w.num_kv_heads):
                first = base_blk[b_, c] + h_ * run_blk[b_, c]
                want[first:first + used_blk[b_, c]] = share       # blocks that are only room to grow belong to nobody
        assert np.array_equal(phys[c], want)

    rng = np.random.default_rng(seed)
    seen = np.zeros(2 * h["gblocks"], dtype=np.int32)       # per unit
    pid_owner = {}
    members = {}
    for it in range(P):
        members.setdefault(int(recs[it, 12]), []).append(it)
    cost = np.zeros(P, dtype=np.int64)
    pool_cost = 0
    for gi in range(NG):
        ngran, pseg0, nps, nworkers, counter = groups[gi, :5]
        ws = sorted(members.get(gi, []), key=lambda x: int(recs[x, 13]) & 0xffff)
        assert len(ws) == nworkers and [int(recs[x, 13]) & 0xffff for x in ws] == list(range(nworkers))
        assert all(recs[x, 13] >> 16 == nps and recs[x, 14] == ngran and recs[x, 15] == pseg0 for x in ws)
        assert 0 <= nps <= 32 and counter == gi
        if h["work_rep"] > 4:
            assert ngran == 0                                # two waves on the same blocks: static split only
        # tickets are handed out in ascending order to whichever worker asks next
        hand = sorted(rng.integers(0, nworkers, size=ngran).tolist()) if ngran else []
        tickets = {r: [] for r in range(nworkers)}
        for t, r in zip(range(ngran), rng.permutation(hand) if ngran else []):
            tickets[int(r)].append(t)
        if nps:
            assert psegs[pseg0, 3] == 0
            last = psegs[pseg0 + nps - 1]
            J = ITER_UNITS[segs[last[0], 2]]
            assert last[3] + (last[2] + J - 1) // J == ngran
        for r, it in enumerate(ws):
            g0, g1, s, pid = recs[it, :4]
            if g0 < g1:
                assert recs[it, 4:12].tolist() == segs[s].tolist()
            last_seg, used = -1, set()
            u, u1 = 2 * g0, 2 * g1
            while u < u1:                                    # own range
                b_, h_, cls, ntok, blk0, nblk, gblk0, spid = segs[s]
                bh = b_ * h["work_heads"] + h_
                if u >= 2 * (gblk0 + nblk):
                    s += 1
                    pid = segs[s, 7]                         # enters the next segment as its first visitor
                    continue
                assert 2 * gblk0 <= u
                if s != last_seg:
                    assert pid not in pid_owner
                    pid_owner[pid] = (cls, bh, 0)
                    last_seg = s
                end = min(u1, 2 * (gblk0 + nblk))
                nu = min(ITER_UNITS[cls], end - u)
                seen[u:u + nu] += 1
                cost[it] += nu * h["block_bytes"][cls]
                u += nu
            for t in tickets[r]:                             # pool
                pi = max(i for i in range(nps) if psegs[pseg0 + i, 3] <= t)
                seg, unit0, nunits, gran0, slot0 = psegs[pseg0 + pi, :5]
                b_, h_, cls, ntok, blk0, nblk, gblk0, spid = segs[seg]
                bh = b_ * h["work_heads"] + h_
                J = ITER_UNITS[cls]
                us = unit0 + (t - gran0) * J
                nu = min(J, unit0 + nunits - us)
                assert 0 < nu and us + nu <= 2 * nblk and seg >= last_seg
                if seg != last_seg:
                    slot = slot0 + r
                    assert r < psegs[pseg0 + pi, 5], "a rank that can enter this part from outside has a slot"
                    assert slot not in pid_owner
                    pid_owner[slot] = (cls, bh, 1)
                    used.add(pi)
                    last_seg = seg
                seen[2 * gblk0 + us:2 * gblk0 + us + nu] += 1
                pool_cost += nu * h["block_bytes"][cls]
            for pi in range(nps):                            # slots the worker fills with the neutral state
                if pi not in used and r < psegs[pseg0 + pi, 5]:
                    seg, slot0 = psegs[pseg0 + pi, 0], psegs[pseg0 + pi, 4]
                    assert slot0 + r not in pid_owner
                    pid_owner[slot0 + r] = (segs[seg, 2], segs[seg, 0] * h["work_heads"] + segs[seg, 1], 1)
    assert (seen == 1).all()
    assert sorted(pid_owner) == list(range(h["partials"])) and h["partials"] == plan.sizes.num_partials
    assert bh_off[0] == 0 and bh_off[BH] == h["partials"] and (np.diff(bh_off) >= 0).all()
    for bh in range(BH):
        assert all(pid_owner[p][1] == bh for p in range(bh_off[bh], bh_off[bh + 1]))
    # workspace: the partial states (header + head_dim floats each), then one status word per (sequence, query head)
    assert h["ws_status_off"] == max(h["partials"], 1) * h["work_rep"] * (w.head_dim + header_floats) * 4
    assert plan.sizes.workspace_bytes == h["ws_status_off"] + (4 * w.batch * w.num_q_heads + 15) // 16 * 16
    return h, cost, pool_cost


@pytest.mark.parametrize("cfg,workers", [(1, 64), (1, 2048), (2, 2048), (3, 512), (4, 2048), (5, 512), (5, 7)])
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
    for c in range(_lib.NUM_CLASSES):
        blocks = sum(((int(plan.class_tokens[b, c]) + 63) // 64) * w.num_kv_heads for b in range(w.batch))
        assert plan.sizes.class_blocks[c] == blocks
        assert plan.sizes.class_bytes[c] == blocks * O.block_bytes(c, w.head_dim, w.group_size)
    h, cost, pool_cost = _check_work_split(plan, w, workers)
    if cfg == 4:
        # the headline shape has pools: a fifth of the bytes, the rest in near-equal own ranges
        total = cost.sum() + pool_cost
        assert 0.15 * total <= pool_cost <= 0.25 * total and h["groups"] == 256   # long ranges: groups of eight


@pytest.mark.parametrize("env", [{"COCKTAIL_POOL_PERCENT": "100"}, {"COCKTAIL_POOL_PERCENT": "0"},
                                 {"COCKTAIL_GROUP_WORKERS": "3", "COCKTAIL_POOL_PERCENT": "50"},
                                 {"COCKTAIL_LAYOUT": "1"}, {"COCKTAIL_LAYOUT": "1", "COCKTAIL_PAIR_MODE": "2"},
                                 {"COCKTAIL_PAIR_MODE": "3", "COCKTAIL_GROUP_WORKERS": "4"}])
def test_work_split_under_tuning_knobs(env, monkeypatch):
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    for cfg, workers in ((2, 2048), (4, 2048), (1, 64)):
        w = workloads.config(cfg)
        plan, _ = _plan(w, workers)
        _check_work_split(plan, w, workers)


@pytest.mark.parametrize("seed", range(6))
def test_work_split_of_random_small_shapes(seed):
    rng = np.random.default_rng(1000 + seed)
    batch = int(rng.integers(1, 5))
    hkv = int(rng.integers(1, 4))
    chunk = int(rng.choice([8, 16, 64, 128]))
    lens = [int(x) for x in rng.integers(0, 6000, size=batch)]
    w = workloads.small(f"rand{seed}", batch, hkv, hkv, lens, chunk, int(rng.choice([32, 64, 128])), seed_offset=seed)
    for workers in (1, 3, 16, 40):
        plan, _ = _plan(w, workers)
        _check_work_split(plan, w, workers, seed)


def test_plan_handles_empty_sequences_and_tail_only():
    sh = ck.make_shape(3, 2, 2, 128, 16, 32)
    plan = ck.cocktail_plan(sh, [0, 5, 16], [4], 8)
    assert plan.class_tokens.tolist() == [[0, 0, 0, 0], [0, 0, 0, 5], [0, 16, 0, 0]]
    assert list(plan.sizes.class_blocks) == [0, 2, 0, 2] and plan.sizes.num_partials >= 4


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
    sh192 = ck.make_shape(1, 2, 2, 192, 8, 32)        # the planner takes any multiple of 64, the kernels 64 and 128
    p192 = ck.cocktail_plan(sh192, [16], [2, 4], 4)
    cache.plan_host = p192.blob.ctypes.data
    assert L.cocktail_decode_attention(C.byref(sh192), 16, C.byref(cache), 0.0, 16, None, 16, 1 << 20, None) == _lib.EUNSUPPORTED
    assert L.cocktail_reorder_quantize(C.byref(sh192), 16, 16, 0, 0, 0, 192, C.byref(cache), None) == _lib.EUNSUPPORTED
    sh_wide = ck.make_shape(1, 128, 1, 128, 8, 32)        # 128 query heads on one kv head: beyond COCKTAIL_MAX_Q_PER_KV
    p_wide = ck.cocktail_plan(sh_wide, [16], [2, 4], 4)
    cache.plan_host = p_wide.blob.ctypes.data
    assert L.cocktail_decode_attention(C.byref(sh_wide), 16, C.byref(cache), 0.0, 16, None, 16, 1 << 20, None) == _lib.EUNSUPPORTED
    n = C.c_size_t(0)
    assert L.cocktail_stream_read_probe(None, 1 << 30, 16, C.byref(n), None) == _lib.EINVAL
    assert L.cocktail_stream_read_probe(8, 1 << 30, 16, C.byref(n), None) == _lib.EALIGN
    assert L.cocktail_stream_read_probe(16, 1 << 20, 16, C.byref(n), None) == _lib.EINVAL


def test_paged_source_is_validated_on_the_host():
    sh = ck.make_shape(2, 2, 2, 128, 8, 32)
    plan = ck.cocktail_plan(sh, [100, 40], [2, 4] * 6 + [16] * 5, 4)
    L = _lib.lib()
    cache = _lib.Cache()
    cache.plan_host = plan.blob.ctypes.data
    cache.plan_dev = 4096
    ok = dict(k_pages=4096, v_pages=4096, page_table=4096, table_stride=7, page_size=16, num_pages=20, reserved=0,
              stride_page=2 * 16 * 128, stride_h=16 * 128, stride_t=128)

    def call(**kw):
        src = _lib.PagedSource(**{**ok, **kw})
        return L.cocktail_reorder_quantize_paged(C.byref(sh), C.byref(src), C.byref(cache), None)

    assert call(table_stride=6) == _lib.EINVAL and b"page table row" in L.cocktail_last_error()   # 100 tokens = 7 pages
    assert call(page_size=0) == _lib.EINVAL
    assert call(num_pages=0) == _lib.EINVAL
    assert call(k_pages=None) == _lib.EINVAL
    assert call(page_table=None) == _lib.EINVAL
    assert call(v_pages=4104) == _lib.EALIGN
    assert call(stride_t=100) == _lib.EINVAL
    assert call(stride_h=4) == _lib.EINVAL
    assert call(reserved=1) == _lib.EINVAL
    assert call() == _lib.EINVAL and b"cache buffer" in L.cocktail_last_error()      # geometry accepted, class buffers are NULL
    assert L.cocktail_reorder_quantize_paged(C.byref(sh), None, C.byref(cache), None) == _lib.EINVAL
    assert L.cocktail_reorder_quantize(C.byref(sh), 16, 16, 2, 0, 0, 128, C.byref(cache), None) == _lib.EINVAL


def test_append_capacity_sizes_and_validation():
    w = workloads.config(1)
    sh = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = np.concatenate(workloads.chunk_bits(w))
    p0 = ck.cocktail_plan(sh, w.seq_lens, bits, 64)
    p1 = ck.cocktail_plan(sh, w.seq_lens, bits, 64, append_capacity=130)
    assert p0.sizes.append_capacity == 0 and p0.sizes.append_bytes == 0
    assert p1.sizes.append_capacity == 130
    assert p1.sizes.append_bytes == w.batch * w.num_kv_heads * 3 * 64 * 256     # 3 blocks of 64 fp16 rows per head
    # one more partial per (sequence, kv head), at the end of its range
    assert p1.sizes.num_partials == p0.sizes.num_partials + w.batch * w.num_kv_heads
    _check_work_split(p0, w, 64)
    h = _parse(p1)
    bh_off = _arr(p1.blob, h["off"]["bh_off"], np.int32, w.batch * w.num_kv_heads + 1)
    bh_off0 = _arr(p0.blob, _parse(p0)["off"]["bh_off"], np.int32, w.batch * w.num_kv_heads + 1)
    assert (np.diff(bh_off) == np.diff(bh_off0) + 1).all()
    L = _lib.lib()
    sizes = _lib.Sizes()
    lp = np.asarray(w.seq_lens, np.int32).ctypes.data_as(C.POINTER(C.c_int32))
    bp = bits.ctypes.data_as(C.POINTER(C.c_uint8))
    bad = _lib.PlanOptions(-1, 0)
    assert L.cocktail_plan_ex(C.byref(sh), lp, bp, 4, C.byref(bad), C.byref(sizes), None, 0, None, None) == _lib.EINVAL
    for field in (0, 1, "reserved0"):
        bad = _lib.PlanOptions(0, 0)
        if field == "reserved0":
            bad.reserved0 = 1
        else:
            bad.reserved[field] = 1
        assert L.cocktail_plan_ex(C.byref(sh), lp, bp, 4, C.byref(bad), C.byref(sizes), None, 0, None, None) == _lib.EINVAL
    assert L.cocktail_plan_ex(C.byref(sh), lp, bp, 4, None, C.byref(sizes), None, 0, None, None) == _lib.OK
    w4 = workloads.config(4)
    sh4 = ck.make_shape(w4.batch, w4.num_q_heads, w4.num_kv_heads, w4.head_dim, w4.chunk_size, w4.group_size)
    bits4 = np.concatenate(workloads.chunk_bits(w4))
    assert _parse(ck.cocktail_plan(sh4, w4.seq_lens, bits4, 2048))["pool_segs"] > 0
    assert _parse(ck.cocktail_plan(sh4, w4.seq_lens, bits4, 2048, reproducible=True))["pool_segs"] == 0
    cache = _lib.Cache()
    cache.plan_host = p0.blob.ctypes.data
    assert L.cocktail_append_fp16(C.byref(sh), 16, 16, C.byref(cache), 0, None) == _lib.EINVAL   # no append buffers
    cache.plan_host = p1.blob.ctypes.data
    assert L.cocktail_append_fp16(C.byref(sh), 16, 16, C.byref(cache), 0, None) == _lib.EINVAL   # NULL buffers
    cache.k_app, cache.v_app = 4096, 4096
    assert L.cocktail_append_fp16(C.byref(sh), 16, 16, C.byref(cache), 130, None) == _lib.EINVAL
    assert L.cocktail_append_fp16(C.byref(sh), 16, 16, C.byref(cache), -1, None) == _lib.EINVAL
    assert L.cocktail_append_fp16(C.byref(sh), 8, 16, C.byref(cache), 0, None) == _lib.EALIGN
    assert L.cocktail_append_fp16(C.byref(sh), None, 16, C.byref(cache), 0, None) == _lib.EINVAL
    # decode: num_appended must fit the plan
    cache.plan_dev = 4096
    cache.num_appended = 131
    assert L.cocktail_decode_attention(C.byref(sh), 16, C.byref(cache), 0.0, 16, None, 16, 1 << 30, None) == _lib.EINVAL
    cache.plan_host = p0.blob.ctypes.data
    cache.num_appended = 1
    assert L.cocktail_decode_attention(C.byref(sh), 16, C.byref(cache), 0.0, 16, None, 16, 1 << 30, None) == _lib.EINVAL
    big = ck.make_shape(1, 1, 1, 128, 64, 32)
    with pytest.raises(ck.CocktailError) as e:
        ck.cocktail_plan(big, [1 << 24], np.full((1 << 24) // 64, 2, np.uint8), 4)
    assert e.value.code == _lib.EUNSUPPORTED


def test_chunk_bitwidths_validates_on_host():
    L = _lib.lib()
    args = (4096, 4096, 4096, 0.6, 0.1, 4096, 4096, None)   # chunk_off, query, chunks, alpha, beta, scores, bits, stream
    assert L.cocktail_chunk_bitwidths(0, 768, 10, *args) == _lib.EINVAL
    assert L.cocktail_chunk_bitwidths(1, 0, 10, *args) == _lib.EINVAL
    assert L.cocktail_chunk_bitwidths(1, 768, -1, *args) == _lib.EINVAL
    assert L.cocktail_chunk_bitwidths(1, 768, 10, 4096, 4096, 4096, 1.5, 0.1, 4096, 4096, None) == _lib.EINVAL
    assert L.cocktail_chunk_bitwidths(1, 768, 10, 4096, 4096, 4096, 0.6, -0.1, 4096, 4096, None) == _lib.EINVAL
    assert L.cocktail_chunk_bitwidths(1, 768, 10, None, 4096, 4096, 0.6, 0.1, 4096, 4096, None) == _lib.EINVAL
    assert L.cocktail_chunk_bitwidths(1, 768, 10, 4096, 4096, None, 0.6, 0.1, 4096, 4096, None) == _lib.EINVAL
    assert L.cocktail_chunk_bitwidths(1, 768, 10, 4096, 4098, 4096, 0.6, 0.1, 4096, 4096, None) == _lib.EALIGN
    assert L.cocktail_chunk_bitwidths(1, 768, 0, 4096, 4096, None, 0.6, 0.1, None, None, None) == _lib.OK   # nothing to do
    assert L.cocktail_selftest_arithmetic(None, None) == _lib.EINVAL
    assert L.cocktail_selftest_arithmetic(4, None) == _lib.EALIGN


@pytest.mark.parametrize("rep,quads,valu", [(1, False, False), (2, True, False), (3, True, False), (4, True, False), (5, True, False),
                                            (8, True, False), (12, True, False), (16, True, False), (11, False, False), (4, False, True), (8, False, True)])
def test_v_layout_follows_the_query_to_kv_head_ratio(rep, quads, valu):
    """Token quads where a wave serves four query heads of a kv head (ratios 2 to 8); one-wave workgroups get pools.
    Vector-ALU-only plans and ratios beyond 8 run one query head per wave: token rows, a work head per query head."""
    shape = ck.make_shape(2, 2 * rep, 2, 128, 64, 32)
    bits = np.array([2, 4, 16, 2] * 16 + [4, 2] * 16, dtype=np.uint8)
    plan = ck.cocktail_plan(shape, [64 * 64, 32 * 64], bits, 16, vector_alu_only=valu)
    assert int(plan.sizes.v_layout) == int(quads)
    h = _parse(plan)
    assert h["rep"] == rep and h["v_layout"] == int(quads)
    work_rep = {12: 6, 16: 8}.get(rep, rep) if quads else 1      # sets of query heads that read a kv head's blocks together
    assert h["work_heads"] == 2 * rep // work_rep and h["work_rep"] == work_rep
    groups = _arr(plan.blob, h["off"]["group_rec"], np.int32, 8 * h["groups"]).reshape(-1, 8)
    assert (groups[:, 0] > 0).any() == (h["work_rep"] <= 4)
    w = workloads.small("vl", 2, 2 * rep, 2, [64 * 64, 32 * 64], 64, 32)
    _check_work_split(plan, w, 16)


def test_room_to_grow_keeps_the_cache_layout_from_plan_to_plan():
    """cocktail_plan_options::max_seq_lens: FP16 runs are laid out for the length a sequence may reach, so the plan
    of a longer context (more FP16 tokens at the end, Sec. III-A) describes the same buffers."""
    w = workloads.small("grow", 3, 4, 2, [300, 64, 1000], 32, 32, mix=(0.2, 0.4, 0.4), seed_offset=41)
    sh = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = workloads.chunk_bits(w)
    flat = np.concatenate(bits)
    most = [300 + 500, 64, 1000 + 70]
    plain = ck.cocktail_plan(sh, w.seq_lens, flat, 64, append_capacity=512)
    p0 = ck.cocktail_plan(sh, w.seq_lens, flat, 64, append_capacity=512, max_seq_lens=most)
    nc = _lib.NUM_CLASSES
    f = ck.cocktail_plan_field

    def layout(plan):
        base = _arr(plan.blob, f(plan, "off_blk_base"), np.int32, nc * (w.batch + 1)).reshape(w.batch + 1, nc)
        run = _arr(plan.blob, f(plan, "off_run_blocks"), np.int32, nc * w.batch).reshape(w.batch, nc)
        used = _arr(plan.blob, f(plan, "off_nblk"), np.int32, nc * w.batch).reshape(w.batch, nc)
        return base, run, used

    base, run, used = layout(p0)
    base_plain, run_plain, used_plain = layout(plain)
    assert np.array_equal(used, used_plain) and np.array_equal(run_plain, used_plain)      # without room: run = used blocks
    assert np.array_equal(run[:, :3], used[:, :3])                                          # only FP16 runs get room
    for b in range(w.batch):
        n16 = int(p0.class_tokens[b, 3])
        assert run[b, 3] == -(-(n16 + most[b] - w.seq_lens[b]) // 64)
    assert np.array_equal(np.diff(base, axis=0), run * w.num_kv_heads)
    assert [int(x) for x in p0.sizes.class_blocks] == [int(x) for x in base[-1]]
    assert int(p0.sizes.packed_bytes) == int(plain.sizes.packed_bytes)                      # algorithmic bytes: tokens only
    # (the replay of the work split does not know the partial ids of the append workgroups: plans without them)
    _check_work_split(ck.cocktail_plan(sh, w.seq_lens, flat, 64, max_seq_lens=most), w, 64)
    # a later plan: sequence 0 grew by 200 tokens (6 chunks completed, all FP16), sequence 2 by 70
    longer = [500, 64, 1070]
    bits1 = [np.concatenate([bits[b], np.full(longer[b] // 32 - len(bits[b]), 16, np.uint8)]) for b in range(3)]
    p1 = ck.cocktail_plan(sh, longer, np.concatenate(bits1), 64, append_capacity=512, max_seq_lens=most)
    base1, run1, used1 = layout(p1)
    assert np.array_equal(base1, base) and np.array_equal(run1, run)
    assert [int(x) for x in p1.sizes.class_bytes] == [int(x) for x in p0.sizes.class_bytes]
    assert np.array_equal(p1.class_tokens[:, :3], p0.class_tokens[:, :3])
    assert (p1.class_tokens[:, 3] - p0.class_tokens[:, 3]).tolist() == [200, 0, 70]
    _check_work_split(ck.cocktail_plan(sh, longer, np.concatenate(bits1), 64, max_seq_lens=most),
                      w.__class__(**{**w.__dict__, "seq_lens": tuple(longer)}), 64)
    # validation
    with pytest.raises(ck.CocktailError, match="below seq_lens"):
        ck.cocktail_plan(sh, w.seq_lens, flat, 64, max_seq_lens=[299, 64, 1000])
    with pytest.raises(ValueError):
        ck.cocktail_plan(sh, w.seq_lens, flat, 64, max_seq_lens=[300, 64])


def test_fold_rejects_plans_that_do_not_belong_together():
    """Host-side checks of cocktail_fold_appended (no kernel is launched on any of these paths)."""
    w = workloads.small("foldv", 2, 2, 2, [100, 40], 16, 32, mix=(0.2, 0.4, 0.4), seed_offset=43)
    sh = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = [np.array([4, 2, 2, 16, 2, 2], np.uint8), np.array([2, 16], np.uint8)]   # 16 INT4 tokens: one more chunk fits its block
    most = [200, 140]
    L = _lib.lib()

    def plan(lens, bit_lists, **kw):
        return ck.cocktail_plan(sh, lens, np.concatenate(bit_lists), 16, **kw)

    def grown(lens):
        return [np.concatenate([bits[b], np.full(lens[b] // 16 - len(bits[b]), 16, np.uint8)]) for b in range(2)]

    p0 = plan(w.seq_lens, bits, append_capacity=64, max_seq_lens=most)
    good = plan([110, 50], grown([110, 50]), append_capacity=64, max_seq_lens=most)
    desc = _lib.Cache()
    desc.plan_host = p0.blob.ctypes.data
    fake = 1 << 20                               # never dereferenced: every call below fails validation first
    desc.plan_dev = fake
    desc.k_app = desc.v_app = fake
    desc.k[3] = desc.v[3] = fake
    desc.num_appended = 10

    def fold(new_plan, new_dev=fake):
        return L.cocktail_fold_appended(C.byref(sh), C.byref(desc), new_plan.blob.ctypes.data if new_plan else None, new_dev, None)

    assert fold(None) == _lib.EINVAL
    assert fold(good, None) == _lib.EINVAL
    assert fold(good, fake + 4) == _lib.EALIGN
    # a different layout (planned without room to grow), fewer tokens than before, more than the append buffers hold
    assert fold(plan([110, 50], grown([110, 50]), append_capacity=64)) == _lib.EINVAL
    assert b"lays the cache out differently" in L.cocktail_last_error()
    assert fold(plan([90, 40], [bits[0][:5], bits[1]], append_capacity=64, max_seq_lens=most)) == _lib.EINVAL
    assert fold(plan([180, 50], grown([180, 50]), append_capacity=64, max_seq_lens=most)) == _lib.EINVAL
    assert b"append buffers hold" in L.cocktail_last_error()
    # a completed chunk that is not FP16: the new plan differs in more than FP16 tokens at the end
    wrong = grown([116, 50])
    wrong[0][-1] = 4
    assert fold(plan([116, 50], wrong, append_capacity=64, max_seq_lens=most)) == _lib.EINVAL
    assert b"more than FP16 tokens" in L.cocktail_last_error()
    # lockstep counting: every sequence must have grown by num_appended
    assert fold(plan([110, 45], grown([110, 45]), append_capacity=64, max_seq_lens=most)) == _lib.EINVAL
    # a plan without append buffers cannot be folded from
    desc.plan_host = plan(w.seq_lens, bits, max_seq_lens=most).blob.ctypes.data
    assert fold(good) == _lib.EINVAL
