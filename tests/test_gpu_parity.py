"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded inputs.

Bar: packed codes, scales/zeros and the reorder permutation bit-exact; attention outputs
within 2e-3 max relative error per (sequence, query head): max_d |gpu - ref| / max_d |ref|.
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import cocktail_oracle as O
import paper_2503_23294_amd as ck

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


class Case:
    """Runs plan -> reorder_quantize -> decode_attention on the GPU for one workload layer."""

    def __init__(self, w, layer=0, workers=None, sm_scale=0.0, strided_pad=0, vector_alu_only=False):
        self.w, self.layer = w, layer
        dev = _dev()
        self.shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
        self.bits = workloads.chunk_bits(w)
        flat_bits = np.concatenate(self.bits) if self.bits else np.zeros(0, np.uint8)
        if workers is None:
            workers = ck.cocktail_default_workers(self.shape, vector_alu_only)
        self.plan = ck.cocktail_plan(self.shape, w.seq_lens, flat_bits, workers, vector_alu_only=vector_alu_only)
        self.cache = ck.PackedCache(self.plan, dev)
        for t in self.cache.k + self.cache.v:
            t.fill_(0xAB)                       # the library must overwrite padding too
        if strided_pad:
            # padded [B, Hkv, Tmax, D + pad] source
            tmax = max(w.seq_lens)
            st = w.head_dim + strided_pad
            k = np.zeros((w.batch, w.num_kv_heads, tmax, st), dtype=np.float16)
            v = np.zeros_like(k)
            for b in range(w.batch):
                for h in range(w.num_kv_heads):
                    kh, vh = workloads.kv_head(w, layer, b, h)
                    k[b, h, :w.seq_lens[b], :w.head_dim] = kh
                    v[b, h, :w.seq_lens[b], :w.head_dim] = vh
            self.k_dev, self.v_dev = torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev)
            ck.cocktail_reorder_quantize(self.cache, self.k_dev, self.v_dev, stride_b=w.num_kv_heads * tmax * st,
                                         stride_h=tmax * st, stride_t=st)
        else:
            k, v = workloads.kv_flat(w, layer, threads=16)
            self.k_dev, self.v_dev = torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev)
            ck.cocktail_reorder_quantize(self.cache, self.k_dev, self.v_dev, ragged=True)
        self.q = workloads.query(w, layer)
        self.q_dev = torch.from_numpy(self.q).to(dev)
        self.sm_scale = sm_scale
        self.out_dev, self.lse_dev = ck.cocktail_decode_attention(self.cache, self.q_dev, sm_scale)
        torch.cuda.synchronize()
        self.out = self.out_dev.cpu().numpy()
        self.lse = self.lse_dev.cpu().numpy()
        # V is stored in token quads where 2 to 8 query heads share a kv head (unless the plan keeps to the vector ALU)
        self.v_quads = int(self.plan.sizes.v_layout) == 1
        rep = w.num_q_heads // w.num_kv_heads
        assert self.v_quads == (rep >= 2 and not vector_alu_only and rep not in (11, 13))
        self.kbuf = [t.cpu().numpy() for t in self.cache.k]
        self.vbuf = [t.cpu().numpy() for t in self.cache.v]
        ct = self.plan.class_tokens.astype(np.int64)
        self.nblk = (ct + 63) // 64
        self.blk_base = np.zeros((w.batch + 1, O.NUM_CLASSES), dtype=np.int64)
        self.blk_base[1:] = np.cumsum(self.nblk * w.num_kv_heads, axis=0)

    def check_plan(self):
        pos = 0
        for b, t in enumerate(self.w.seq_lens):
            sp = O.plan_sequence(t, self.w.chunk_size, self.bits[b])
            n = t // self.w.chunk_size
            assert self.plan.perm[pos:pos + n].tolist() == sp.perm.tolist()
            assert tuple(self.plan.class_tokens[b]) == sp.class_tokens
            pos += n

    def check_head(self, b, h):
        """Bit-exact cache bytes of kv head (b, h) and attention parity of its query heads."""
        w = self.w
        kh, vh = workloads.kv_head(w, self.layer, b, h)
        oc = O.reorder_quantize([kh[None]], [vh[None]], [self.bits[b]], w.chunk_size, w.group_size)
        for c in range(O.NUM_CLASSES):
            bb = O.block_bytes(c, w.head_dim, w.group_size)
            lo = (self.blk_base[b, c] + h * self.nblk[b, c]) * bb
            hi = lo + self.nblk[b, c] * bb
            for which, buf in (("k", self.kbuf[c]), ("v", self.vbuf[c])):
                ref = O.pack_class_buffer(oc, c, which, v_quads=self.v_quads)
                got = buf[lo:hi]
                assert ref.size == got.size
                if not np.array_equal(ref, got):
                    bad = np.flatnonzero(ref != got)
                    raise AssertionError(f"cache bytes differ: b={b} h={h} class={c} {which}: {bad.size} bytes, "
                                         f"first at {bad[0]} (block {bad[0] // bb}, offset {bad[0] % bb})")
        rep = w.num_q_heads // w.num_kv_heads
        sm = self.sm_scale if self.sm_scale > 0 else None
        worst = 0.0
        for r in range(rep):
            hq = h * rep + r
            ref, rl = O.decode_attention(self.q[b:b + 1, hq:hq + 1], oc, sm_scale=sm)
            ref, rl = ref[0, 0], rl[0, 0]
            got = self.out[b, hq].astype(np.float64)
            if w.seq_lens[b] == 0:
                assert (got == 0).all() and np.isneginf(self.lse[b, hq])
                continue
            err = np.abs(got - ref).max() / np.abs(ref).max()
            worst = max(worst, err)
            assert err <= TOL, f"attention b={b} hq={hq}: max rel err {err:.3e}"
            assert abs(self.lse[b, hq] - rl) <= 1e-4 * max(1.0, abs(rl)), (self.lse[b, hq], rl)
        return worst

    def check_all(self):
        self.check_plan()
        worst = 0.0
        for b in range(self.w.batch):
            for h in range(self.w.num_kv_heads):
                worst = max(worst, self.check_head(b, h))
        return worst


def _announce(msg):
    print(f"[parity] {msg}", flush=True)


@pytest.mark.parametrize("workers", [None, 1, 7, 64])
def test_config1_all_heads(workers):
    _announce(f"config 1 workers={workers}")
    c = Case(workloads.config(1), workers=workers)
    worst = c.check_all()
    _announce(f"config 1 worst rel err {worst:.2e}")


@pytest.mark.parametrize("group", [32, 64, 128])
@pytest.mark.parametrize("rep", [1, 2, 3, 4, 5, 6, 7, 8, 11, 12, 16])
def test_group_sizes_and_gqa(group, rep):
    w = workloads.small(f"g{group}_r{rep}", 2, 2 * rep, 2, [64 * 5 + 32 * 3 + 7, 32 * 9], 32, group,
                        mix=(0.2, 0.25, 0.25, 0.3), seed_offset=group + rep)
    _announce(w.name)
    Case(w, workers=5).check_all()


@pytest.mark.parametrize("rep,head_dim,workers", [(2, 128, 5), (4, 128, 16), (8, 128, 7), (4, 64, 9), (16, 64, 12)])
def test_grouped_queries_on_the_vector_alu_only(rep, head_dim, workers):
    """A plan made with vector_alu_only runs grouped-query shapes on the kernel without matrix instructions: one
    query head per wave, V in token rows, pools as with one head per kv head.  Same cache bytes for K, same answers."""
    w = workloads.small(f"valu_r{rep}_d{head_dim}", 3, 2 * rep, 2, [3000, 700, 64 * 5 + 9], 64, 32,
                        mix=(0.2, 0.2, 0.2, 0.4), head_dim=head_dim, seed_offset=700 + rep)
    _announce(w.name)
    c = Case(w, workers=workers, vector_alu_only=True)
    assert ck.cocktail_plan_field(c.plan, "work_heads") == w.num_q_heads and ck.cocktail_plan_field(c.plan, "work_rep") == 1
    c.check_all()
    ck.cocktail_decode_check(c.cache)
    ref = Case(w, workers=workers)                           # the default plan (matrix instructions up to ratio 8)
    assert (c.out.astype(np.float32) - ref.out.astype(np.float32)).__abs__().max() <= 2e-3 * np.abs(ref.out.astype(np.float32)).max()


@pytest.mark.parametrize("group", [32, 64])
@pytest.mark.parametrize("rep", [1, 2, 3, 4, 5, 8, 12])
def test_head_dim_64(group, rep):
    """head_dim 64: a lane still works on 64 channels, so a wave takes 64 tokens at a time instead of 32."""
    w = workloads.small(f"d64_g{group}_r{rep}", 2, 2 * rep, 2, [64 * 5 + 32 * 3 + 7, 64 * 9 + 1], 32, group,
                        mix=(0.2, 0.25, 0.25, 0.3), head_dim=64, seed_offset=64 + group + rep)
    _announce(w.name)
    Case(w, workers=5).check_all()


@pytest.mark.parametrize("rep,workers", [(1, 24), (4, 7)])
def test_head_dim_64_long_sequences_with_pools(rep, workers):
    w = workloads.small(f"d64pools_r{rep}", 3, 2 * rep, 2, [6000, 2500, 9000], 64, 32, mix=(0.2, 0.2, 0.2, 0.4),
                        head_dim=64, seed_offset=164 + rep)
    _announce(w.name)
    c = Case(w, workers=workers)
    assert _counters(c)[1] > 0, "this shape is meant to exercise the pools"
    c.check_all()
    ck.cocktail_decode_check(c.cache)


@pytest.mark.parametrize("mix", [(1, 0, 0), (0, 1, 0), (0, 0, 1), (0.5, 0, 0.5), (0, 1, 0, 0), (0.3, 0.3, 0, 0.4),
                                 (0, 0.5, 0.5, 0), (0.25, 0.25, 0.25, 0.25)])
def test_single_class_and_missing_class(mix):
    w = workloads.small("mix" + "".join(str(int(10 * m)) for m in mix), 1, 2, 2, [8 * 40 + 3], 8, 32, mix=mix,
                        seed_offset=11)
    _announce(w.name)
    Case(w, workers=3).check_all()


def test_ragged_batch_with_empty_and_tail_only_sequences():
    w = workloads.small("ragged_edge", 5, 4, 2, [0, 5, 96 * 7 + 50, 64, 96], 96, 64, mix=(0.3, 0.3, 0.4),
                        seed_offset=5)
    _announce(w.name)
    c = Case(w, workers=9)
    c.check_all()
    assert (c.out[0] == 0).all()


def test_chunk_smaller_than_block_and_custom_scale():
    w = workloads.small("chunk8", 2, 2, 1, [8 * 77 + 1, 8 * 13], 8, 32, mix=(0.2, 0.4, 0.4), seed_offset=3)
    _announce(w.name)
    Case(w, workers=16, sm_scale=0.05).check_all()


def test_strided_padded_source():
    w = workloads.small("strided", 2, 2, 2, [300, 128], 32, 32, seed_offset=9)
    _announce(w.name)
    Case(w, workers=4, strided_pad=8).check_all()


def test_strided_source_into_a_cache_with_room_to_grow():
    """Dense [B, Hkv, Tmax, D] source, FP16 runs laid out for longer contexts: class buffers equal the oracle's
    image with zero blocks behind every FP16 run, and attention is unaffected by the spare blocks."""
    w = workloads.small("strided_room", 3, 4, 2, [300, 0, 129], 32, 64, mix=(0.3, 0.3, 0.4), seed_offset=19)
    _announce(w.name)
    dev = _dev()
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = workloads.chunk_bits(w)
    room = [65, 130, 1]
    plan = ck.cocktail_plan(shape, w.seq_lens, np.concatenate(bits), 16, max_seq_lens=[t + r for t, r in zip(w.seq_lens, room)])
    cache = ck.PackedCache(plan, dev)
    for t in cache.k + cache.v:
        t.fill_(0xAB)
    tmax = max(w.seq_lens)
    k = np.zeros((w.batch, w.num_kv_heads, tmax, w.head_dim), dtype=np.float16)
    v = np.zeros_like(k)
    ks, vs = [], []
    for b in range(w.batch):
        kh, vh = zip(*[workloads.kv_head(w, 0, b, h) for h in range(w.num_kv_heads)])
        ks.append(np.stack(kh)), vs.append(np.stack(vh))
        k[b, :, :w.seq_lens[b]], v[b, :, :w.seq_lens[b]] = ks[b], vs[b]
    ck.cocktail_reorder_quantize(cache, torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev))
    oc = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    v_quads = int(plan.sizes.v_layout) == 1
    for c in range(O.NUM_CLASSES):
        assert np.array_equal(cache.k[c].cpu().numpy(), O.pack_class_buffer(oc, c, "k", reserve=room)), f"K class {c}"
        assert np.array_equal(cache.v[c].cpu().numpy(), O.pack_class_buffer(oc, c, "v", v_quads=v_quads, reserve=room)), f"V class {c}"
    q = workloads.query(w, 0)
    out, lse = ck.cocktail_decode_attention(cache, torch.from_numpy(q).to(dev))
    ck.cocktail_decode_check(cache)
    ref, _ = O.decode_attention(q, oc)
    got = out.cpu().numpy().astype(np.float64)
    for b in (0, 2):
        err = np.abs(got[b] - ref[b]).max(axis=1) / np.abs(ref[b]).max(axis=1)
        assert err.max() <= TOL
    assert (got[1] == 0).all() and np.isneginf(lse.cpu().numpy()[1]).all()


@pytest.mark.parametrize("page_size,head_major,rep,head_dim,room", [(16, True, 1, 128, 0), (64, False, 1, 128, 0), (128, True, 4, 128, 0),
                                                                    (5, True, 1, 128, 0), (256, False, 2, 128, 0), (16, True, 4, 64, 0),
                                                                    (16, True, 1, 128, 100), (5, False, 4, 128, 70), (64, True, 2, 64, 1)])
def test_paged_source(page_size, head_major, rep, head_dim, room):
    """Reorder+quantize straight from a paged KV cache with a shuffled page table: the packed cache must be the
    one the oracle makes from the gathered K and V, byte for byte.  room: the FP16 runs are laid out with room for
    that many more tokens per sequence (the empty sequence too), which reorder+quantize writes as zero blocks."""
    w = workloads.small(f"paged{page_size}", 3, 2 * rep, 2, [64 * 9 + 21, 0, 700], 32, 32, mix=(0.2, 0.4, 0.4),
                        head_dim=head_dim, seed_offset=600 + page_size)
    _announce(f"{w.name} head_major={head_major} rep={rep}")
    dev = _dev()
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = workloads.chunk_bits(w)
    plan = ck.cocktail_plan(shape, w.seq_lens, np.concatenate(bits), 8,
                            max_seq_lens=[t + room for t in w.seq_lens] if room else None)
    cache = ck.PackedCache(plan, dev)
    for t in cache.k + cache.v:
        t.fill_(0xAB)
    rng = np.random.default_rng(page_size)
    need = [(t + page_size - 1) // page_size for t in w.seq_lens]
    num_pages = sum(need) + 5
    ids = rng.permutation(num_pages)
    table = np.full((w.batch, max(need) + 2), -1, dtype=np.int32)             # entries behind a sequence's pages are not read
    kp = rng.standard_normal((num_pages, w.num_kv_heads, page_size, w.head_dim), dtype=np.float32).astype(np.float16)
    vp = rng.standard_normal((num_pages, w.num_kv_heads, page_size, w.head_dim), dtype=np.float32).astype(np.float16)
    pos = 0
    for b in range(w.batch):
        table[b, :need[b]] = ids[pos:pos + need[b]]
        pos += need[b]
        for h in range(w.num_kv_heads):
            kh, vh = workloads.kv_head(w, 0, b, h)
            for t in range(w.seq_lens[b]):
                kp[table[b, t // page_size], h, t % page_size] = kh[t]
                vp[table[b, t // page_size], h, t % page_size] = vh[t]
    if not head_major:
        kp, vp = np.ascontiguousarray(kp.transpose(0, 2, 1, 3)), np.ascontiguousarray(vp.transpose(0, 2, 1, 3))
    ck.cocktail_reorder_quantize_paged(cache, torch.from_numpy(kp).to(dev), torch.from_numpy(vp).to(dev),
                                       torch.from_numpy(table).to(dev), head_major=head_major)
    torch.cuda.synchronize()
    pools = (kp, vp) if head_major else (kp.transpose(0, 2, 1, 3), vp.transpose(0, 2, 1, 3))
    ks = [O.gather_pages(pools[0], table[b], w.seq_lens[b]) for b in range(w.batch)]
    vs = [O.gather_pages(pools[1], table[b], w.seq_lens[b]) for b in range(w.batch)]
    oc = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    v_quads = int(plan.sizes.v_layout) == 1
    reserve = [room] * w.batch if room else None
    for c in range(O.NUM_CLASSES):
        assert np.array_equal(cache.k[c].cpu().numpy(), O.pack_class_buffer(oc, c, "k", reserve=reserve)), f"K class {c}"
        assert np.array_equal(cache.v[c].cpu().numpy(), O.pack_class_buffer(oc, c, "v", v_quads=v_quads, reserve=reserve)), f"V class {c}"
    q = workloads.query(w, 0)
    out, _ = ck.cocktail_decode_attention(cache, torch.from_numpy(q).to(dev))
    ck.cocktail_decode_check(cache)
    ref, _ = O.decode_attention(q, oc)
    got = out.cpu().numpy().astype(np.float64)
    for b in range(w.batch):
        if w.seq_lens[b]:
            err = np.abs(got[b] - ref[b]).max(axis=1) / np.abs(ref[b]).max(axis=1)
            assert err.max() <= TOL


def test_more_workers_than_blocks_and_repeatability():
    w = workloads.small("tiny", 1, 1, 1, [70], 16, 32, seed_offset=2)
    _announce(w.name)
    c = Case(w, workers=64)
    c.check_all()
    out2, lse2 = ck.cocktail_decode_attention(c.cache, c.q_dev)
    torch.cuda.synchronize()
    assert torch.equal(out2, c.out_dev) and torch.equal(lse2, c.lse_dev)


def _counters(c):
    """The decode kernel's ticket counters inside the device copy of the plan, and the number of pool parts."""
    off, ngroups = ck.cocktail_plan_field(c.plan, "off_counters"), ck.cocktail_plan_field(c.plan, "num_groups")
    stride = ck.cocktail_plan_field(c.plan, "counter_stride_bytes")
    words = c.cache.plan_dev[off:off + stride * ngroups].cpu().numpy().view(np.uint32)[::stride // 4]
    return words, ck.cocktail_plan_field(c.plan, "num_pool_segs")


@pytest.mark.parametrize("workers", [1, 3, 8, 13, 24])
def test_shared_pools_with_few_workers(workers):
    """Few workers on a multi-sequence MHA shape: every group has a pool that spans several segments."""
    w = workloads.small(f"pools{workers}", 3, 2, 2, [3000, 1500, 4500], 64, 32, mix=(0.2, 0.4, 0.4),
                        seed_offset=40 + workers)
    _announce(w.name)
    c = Case(w, workers=workers)
    cnt, pool_segs = _counters(c)
    assert pool_segs > 0, "this shape is meant to exercise the pools"
    assert (cnt == 0).all(), "a call must leave the ticket counters at zero"
    c.check_all()
    for _ in range(3):                       # tickets are handed out anew on every call
        out, lse = ck.cocktail_decode_attention(c.cache, c.q_dev)
        torch.cuda.synchronize()
        assert (_counters(c)[0] == 0).all()
        c.out, c.lse = out.cpu().numpy(), lse.cpu().numpy()
        for b in range(w.batch):
            for h in range(w.num_kv_heads):
                c.check_head(b, h)


@pytest.mark.parametrize("rep,stale", [(1, 3), (1, 1 << 30), (4, 2)])
def test_stale_ticket_counter_is_reported_and_does_not_outlive_the_call(rep, stale):
    """A ticket counter that is not zero when a call starts (an aborted call, overlapping calls) makes the
    workers skip pool pieces.  Such a call must not pass as a result: the rows that miss tokens come out as
    NaN, cocktail_decode_check reports them, and the call after it is sound again."""
    w = workloads.small(f"stale_r{rep}", 3, 2 * rep, 2, [3000, 1500, 4500], 64, 32, mix=(0.2, 0.4, 0.4),
                        seed_offset=140 + rep)
    _announce(f"{w.name} stale={stale}")
    c = Case(w, workers=8)
    c.check_all()
    ck.cocktail_decode_check(c.cache)                        # the call inside Case was sound
    ngroups = ck.cocktail_plan_field(c.plan, "num_groups")
    goff, gsize = ck.cocktail_plan_field(c.plan, "off_group_rec"), ck.cocktail_plan_field(c.plan, "sizeof_group_rec")
    ngran = np.frombuffer(c.plan.blob.tobytes(), dtype=np.int32, count=ngroups * gsize // 4, offset=goff)[::gsize // 4]
    g = int(np.argmax(ngran))
    assert ngran[g] > 3, "this shape is meant to have a pool with several tickets"
    off = ck.cocktail_plan_field(c.plan, "off_counters") + g * ck.cocktail_plan_field(c.plan, "counter_stride_bytes")
    c.cache.plan_dev[off:off + 4] = torch.from_numpy(np.array([stale], dtype=np.uint32).view(np.uint8)).to(c.cache.plan_dev.device)
    out, lse = ck.cocktail_decode_attention(c.cache, c.q_dev)
    with pytest.raises(ck.CocktailError) as e:
        ck.cocktail_decode_check(c.cache)
    assert e.value.code == -6 and "too few" in str(e.value)
    out, lse = out.cpu().numpy().astype(np.float64), lse.cpu().numpy()
    bad_rows = np.isnan(out).all(axis=2)
    assert bad_rows.any() and (np.isnan(out).any(axis=2) == bad_rows).all() and (np.isnan(lse) == bad_rows).all()
    ref = c.out.astype(np.float64)                           # rows that lost no token are results
    good = ~bad_rows
    assert (np.abs(out[good] - ref[good]).max(axis=1) <= TOL * np.abs(ref[good]).max(axis=1)).all()
    assert (_counters(c)[0] == 0).all()                      # the merge put the counters back
    out2, _ = ck.cocktail_decode_attention(c.cache, c.q_dev)
    ck.cocktail_decode_check(c.cache)
    c.out = out2.cpu().numpy()
    for b in range(w.batch):
        for h in range(w.num_kv_heads):
            c.check_head(b, h)


@pytest.mark.parametrize("rep,workers", [(4, 3), (4, 16), (3, 8), (2, 24)])
def test_shared_pools_grouped_query(rep, workers):
    """2 to 4 query heads per kv head run as one wave, so these shapes use the pools too."""
    w = workloads.small(f"gqpools{rep}_{workers}", 3, 2 * rep, 2, [3000, 1500, 4500], 64, 32, mix=(0.2, 0.4, 0.4),
                        seed_offset=90 + rep + workers)
    _announce(w.name)
    c = Case(w, workers=workers)
    cnt, pool_segs = _counters(c)
    assert pool_segs > 0, "this shape is meant to exercise the pools"
    assert (cnt == 0).all(), "a call must leave the ticket counters at zero"
    c.check_all()
    for _ in range(2):
        out, lse = ck.cocktail_decode_attention(c.cache, c.q_dev)
        torch.cuda.synchronize()
        assert (_counters(c)[0] == 0).all()
        c.out, c.lse = out.cpu().numpy(), lse.cpu().numpy()
        for b in range(w.batch):
            for h in range(w.num_kv_heads):
                c.check_head(b, h)


@pytest.mark.parametrize("env", [{"COCKTAIL_POOL_PERCENT": "100"}, {"COCKTAIL_POOL_PERCENT": "0"},
                                 {"COCKTAIL_GROUP_WORKERS": "3", "COCKTAIL_POOL_PERCENT": "50"},
                                 {"COCKTAIL_LAYOUT": "1"}, {"COCKTAIL_LAYOUT": "1", "COCKTAIL_PAIR_MODE": "2"},
                                 {"COCKTAIL_PAIR_MODE": "3", "COCKTAIL_GROUP_WORKERS": "4"},
                                 {"COCKTAIL_COST_WEIGHTS": "1,1,1"}])
def test_planner_tuning_knobs_keep_parity(env, monkeypatch):
    """Every work split the planner can be asked for reads each token exactly once."""
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    w = workloads.small("knobs", 2, 4, 4, [4096, 2304], 128, 64, mix=(0.15, 0.35, 0.5), seed_offset=77)
    _announce(f"{w.name} {env}")
    Case(w, workers=16).check_all()


@pytest.mark.parametrize("rep,capacity,steps,head_dim", [(1, 70, 70, 128), (4, 130, 37, 128), (2, 1, 1, 128), (8, 66, 66, 128),
                                                         (6, 5, 3, 128), (1, 70, 70, 64), (4, 130, 67, 64), (16, 70, 66, 128)])
def test_appended_decode_tokens(rep, capacity, steps, head_dim):
    """Sec. III-A: generated tokens are appended in FP16; every decode step attends to all of them."""
    w = workloads.small(f"append_r{rep}_d{head_dim}", 2, 2 * rep, 2, [64 * 9 + 5, 300], 64, 32, mix=(0.2, 0.4, 0.4),
                        head_dim=head_dim, seed_offset=60 + rep)
    _announce(w.name)
    dev = _dev()
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = workloads.chunk_bits(w)
    plan = ck.cocktail_plan(shape, w.seq_lens, np.concatenate(bits), 12, append_capacity=capacity)
    cache = ck.PackedCache(plan, dev)
    cache.k_app.fill_(0xAB), cache.v_app.fill_(0xAB)       # reorder+quantize must clear the append buffers
    k, v = workloads.kv_flat(w, 0)
    ck.cocktail_reorder_quantize(cache, torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev), ragged=True)
    ks, vs = [], []
    for b in range(w.batch):
        kh, vh = zip(*[workloads.kv_head(w, 0, b, h) for h in range(w.num_kv_heads)])
        ks.append(np.stack(kh)), vs.append(np.stack(vh))
    oc = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    q = workloads.query(w, 0)
    q_dev = torch.from_numpy(q).to(dev)
    rng = np.random.default_rng([workloads.BASE_SEED, 4242, rep])

    def compare():
        out, lse = ck.cocktail_decode_attention(cache, q_dev)
        torch.cuda.synchronize()
        ref, rl = O.decode_attention(q, oc)
        got = out.cpu().numpy().astype(np.float64)
        err = np.abs(got - ref).max(axis=2) / np.abs(ref).max(axis=2)
        assert err.max() <= TOL, f"after {cache.desc.num_appended} appended tokens: max rel err {err.max():.3e}"
        assert np.abs(lse.cpu().numpy() - rl).max() <= 1e-4 * max(1.0, np.abs(rl).max())

    compare()                                               # nothing appended yet
    for step in range(steps):
        kn = rng.standard_normal((w.batch, w.num_kv_heads, w.head_dim), dtype=np.float32).astype(np.float16)
        vn = rng.standard_normal((w.batch, w.num_kv_heads, w.head_dim), dtype=np.float32).astype(np.float16)
        kn[:, :, 3] *= np.float16(6.0)                      # keep the new tokens relevant to the softmax
        ck.cocktail_append_fp16(cache, torch.from_numpy(kn).to(dev), torch.from_numpy(vn).to(dev))
        O.append_tokens(oc, kn, vn)
        if step in (0, 1, 31, 32, 63, 64, steps - 1):
            compare()
    torch.cuda.synchronize()
    assert cache.desc.num_appended == steps
    for which, buf in (("k", cache.k_app), ("v", cache.v_app)):      # append buffers bit-exact, unused rows zero
        assert np.array_equal(buf.cpu().numpy(), O.pack_append_buffer(oc, which, capacity, v_quads=rep >= 2))
    if steps == capacity:
        with pytest.raises(ck.CocktailError):
            ck.cocktail_append_fp16(cache, torch.from_numpy(kn).to(dev), torch.from_numpy(vn).to(dev))


@pytest.mark.parametrize("rep,head_dim,stops", [(1, 128, [40, 0, 700]), (4, 128, [3, 130, 66]), (4, 64, [700, 1, 64]),
                                                (8, 128, [5, 70, 0])])
def test_sequences_that_stop_generating_at_different_steps(rep, head_dim, stops):
    """Sec. III-A in a batch whose sequences generate independently: per-sequence counts on the device, a step
    appends a token to the active sequences only; long runs of appended tokens are shared by several workgroups."""
    w = workloads.small(f"raggedgen_r{rep}_d{head_dim}", 3, 2 * rep, 2, [64 * 9 + 5, 300, 1000], 64, 32,
                        mix=(0.2, 0.4, 0.4), head_dim=head_dim, seed_offset=260 + rep)
    _announce(f"{w.name} stops={stops}")
    dev = _dev()
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = workloads.chunk_bits(w)
    capacity = max(stops)
    plan = ck.cocktail_plan(shape, w.seq_lens, np.concatenate(bits), 12, append_capacity=capacity)
    assert ck.cocktail_plan_field(plan, "append_slices") == -(-(-(-capacity // 64)) // 8)
    cache = ck.PackedCache(plan, dev)
    k, v = workloads.kv_flat(w, 0)
    ck.cocktail_reorder_quantize(cache, torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev), ragged=True)
    ks, vs = [], []
    for b in range(w.batch):
        kh, vh = zip(*[workloads.kv_head(w, 0, b, h) for h in range(w.num_kv_heads)])
        ks.append(np.stack(kh)), vs.append(np.stack(vh))
    oc = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    q = workloads.query(w, 0)
    q_dev = torch.from_numpy(q).to(dev)
    rng = np.random.default_rng([workloads.BASE_SEED, 4343, rep])

    def compare():
        out, lse = ck.cocktail_decode_attention(cache, q_dev)
        ck.cocktail_decode_check(cache)
        ref, rl = O.decode_attention(q, oc)
        got = out.cpu().numpy().astype(np.float64)
        err = np.abs(got - ref).max(axis=2) / np.abs(ref).max(axis=2)
        assert err.max() <= TOL, f"appended {cache.appended.tolist()}: max rel err {err.max():.3e}"
        assert np.abs(lse.cpu().numpy() - rl).max() <= 1e-4 * max(1.0, np.abs(rl).max())

    for step in range(capacity + 2):                        # two steps past the end: nobody is active, nothing changes
        active = np.array([step < s for s in stops], dtype=np.uint8)
        kn = rng.standard_normal((w.batch, w.num_kv_heads, w.head_dim), dtype=np.float32).astype(np.float16)
        vn = rng.standard_normal((w.batch, w.num_kv_heads, w.head_dim), dtype=np.float32).astype(np.float16)
        kn[:, :, 3] *= np.float16(6.0)
        ck.cocktail_append_fp16_ragged(cache, torch.from_numpy(kn).to(dev), torch.from_numpy(vn).to(dev),
                                       torch.from_numpy(active).to(dev))
        O.append_tokens(oc, kn, vn, active)
        if step in (0, 1, 2, 63, 64, 65, 129, 511, 512, capacity - 1, capacity + 1):
            compare()
    assert cache.appended.cpu().tolist() == stops
    v_quads = rep >= 2
    for which, buf in (("k", cache.k_app), ("v", cache.v_app)):      # append buffers bit-exact, unused rows zero
        assert np.array_equal(buf.cpu().numpy(), O.pack_append_buffer(oc, which, capacity, v_quads=v_quads))
    # a full sequence stays as it is when it is asked to take another token
    ck.cocktail_append_fp16_ragged(cache, torch.from_numpy(kn).to(dev), torch.from_numpy(vn).to(dev))
    torch.cuda.synchronize()
    full = [min(s + 1, capacity) for s in stops]
    assert cache.appended.cpu().tolist() == full


@pytest.mark.parametrize("rep,head_dim,ragged", [(1, 128, True), (4, 128, True), (4, 64, False), (8, 128, True), (1, 64, False)])
def test_folding_appended_tokens_into_the_packed_cache(rep, head_dim, ragged):
    """Sec. III-A over a long generation: the appended tokens become context.  After every fold the class buffers
    are, byte for byte, those of a cache built from the longer context (FP16 runs laid out with room to grow), the
    append counts are back to zero, and attention agrees with the oracle before and after."""
    w = workloads.small(f"fold_r{rep}_d{head_dim}", 3, 2 * rep, 2, [64 * 5 + 37, 40, 700], 32, 32,
                        mix=(0.2, 0.4, 0.4), head_dim=head_dim, seed_offset=290 + rep)
    _announce(f"{w.name} ragged={ragged}")
    dev = _dev()
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = [x.copy() for x in workloads.chunk_bits(w)]
    lens = list(w.seq_lens)
    most = [lens[0] + 400, lens[1] + 400, lens[2] + 400]
    capacity = 200
    plan = ck.cocktail_plan(shape, lens, np.concatenate(bits), 12, append_capacity=capacity, max_seq_lens=most)
    cache = ck.PackedCache(plan, dev)
    for t in cache.k + cache.v:
        t.fill_(0xAB)                                       # room to grow has to be written too (as zeros)
    k, v = workloads.kv_flat(w, 0)
    ck.cocktail_reorder_quantize(cache, torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev), ragged=True)
    ks, vs = [], []
    for b in range(w.batch):
        kh, vh = zip(*[workloads.kv_head(w, 0, b, h) for h in range(w.num_kv_heads)])
        ks.append(np.stack(kh)), vs.append(np.stack(vh))
    oc = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    q = workloads.query(w, 0)
    q_dev = torch.from_numpy(q).to(dev)
    rng = np.random.default_rng([workloads.BASE_SEED, 4747, rep, head_dim])
    v_quads = int(plan.sizes.v_layout) == 1

    def compare(what):
        out, lse = ck.cocktail_decode_attention(cache, q_dev)
        ck.cocktail_decode_check(cache)
        ref, rl = O.decode_attention(q, oc)
        got = out.cpu().numpy().astype(np.float64)
        err = np.abs(got - ref).max(axis=2) / np.abs(ref).max(axis=2)
        assert err.max() <= TOL, f"{what}: max rel err {err.max():.3e}"
        assert np.abs(lse.cpu().numpy() - rl).max() <= 1e-4 * max(1.0, np.abs(rl).max())

    def compare_bytes(what):
        reserve = [most[b] - oc.seq_lens[b] for b in range(w.batch)]
        for c in range(O.NUM_CLASSES):
            for which, bufs in (("k", cache.k), ("v", cache.v)):
                ref = O.pack_class_buffer(oc, c, which, v_quads=v_quads, reserve=reserve)
                got = bufs[c].cpu().numpy()
                assert ref.size == got.size, f"{what}: class {c} {which}: {got.size} bytes, {ref.size} expected"
                if not np.array_equal(ref, got):
                    bad = np.flatnonzero(ref != got)
                    bb = O.block_bytes(c, w.head_dim, w.group_size)
                    raise AssertionError(f"{what}: class {c} {which}: {bad.size} bytes differ, first in block {bad[0] // bb} "
                                         f"at offset {bad[0] % bb}")

    compare_bytes("after reorder+quantize")
    compare("before any token")
    # three rounds: generate (sequences stop at different steps when ragged), decode, fold, decode
    for rnd, steps in enumerate(([90, 0, 200], [64, 7, 1], [0, 0, 0])):
        if not ragged:
            steps = [max(steps)] * 3
        for step in range(max(steps)):
            active = np.array([step < n for n in steps], dtype=np.uint8)
            kn = rng.standard_normal((w.batch, w.num_kv_heads, w.head_dim), dtype=np.float32).astype(np.float16)
            vn = rng.standard_normal((w.batch, w.num_kv_heads, w.head_dim), dtype=np.float32).astype(np.float16)
            if ragged:
                ck.cocktail_append_fp16_ragged(cache, torch.from_numpy(kn).to(dev), torch.from_numpy(vn).to(dev),
                                               torch.from_numpy(active).to(dev))
            else:
                ck.cocktail_append_fp16(cache, torch.from_numpy(kn).to(dev), torch.from_numpy(vn).to(dev), step)
            O.append_tokens(oc, kn, vn, active)
        compare(f"round {rnd}, {steps} tokens appended")
        lens = [lens[b] + steps[b] for b in range(w.batch)]
        bits = [np.concatenate([bits[b], np.full(lens[b] // w.chunk_size - len(bits[b]), 16, np.uint8)]) for b in range(w.batch)]
        longer = ck.cocktail_plan(shape, lens, np.concatenate(bits), 12, append_capacity=capacity, max_seq_lens=most)
        assert [int(x) for x in longer.sizes.class_bytes] == [int(x) for x in plan.sizes.class_bytes]
        ck.cocktail_fold_appended(cache, longer)
        O.fold_appended(oc)
        assert oc.seq_lens == lens and all(np.array_equal(oc.bits[b], bits[b]) for b in range(w.batch))
        torch.cuda.synchronize()
        if ragged:
            assert cache.appended.cpu().tolist() == [0, 0, 0]
        assert int(cache.desc.num_appended) == 0
        compare_bytes(f"after fold {rnd}")
        compare(f"after fold {rnd}")
    # generation goes on after a fold: the append buffers start from their first row again
    kn = rng.standard_normal((w.batch, w.num_kv_heads, w.head_dim), dtype=np.float32).astype(np.float16)
    vn = rng.standard_normal((w.batch, w.num_kv_heads, w.head_dim), dtype=np.float32).astype(np.float16)
    if ragged:
        ck.cocktail_append_fp16_ragged(cache, torch.from_numpy(kn).to(dev), torch.from_numpy(vn).to(dev))
    else:
        ck.cocktail_append_fp16(cache, torch.from_numpy(kn).to(dev), torch.from_numpy(vn).to(dev), 0)
    O.append_tokens(oc, kn, vn)
    compare("one more token after the last fold")


@pytest.mark.parametrize("alpha,beta", [(0.6, 0.1), (0.0, 0.0), (0.3, 0.5), (1.0, 1.0)])
def test_chunk_level_quantization_search(alpha, beta):
    """Sec. III-B: scores and bitwidths of every chunk, bit for bit (the arithmetic is fixed on both sides)."""
    num_chunks = [4096, 256, 1, 0, 1000]              # 128K tokens in 32-token chunks, ..., one chunk, none
    _announce(f"search alpha={alpha} beta={beta}")
    q, cs = workloads.embeddings(11, num_chunks)
    cs[4][17] = 0.0                                    # a zero embedding scores 0
    dev = _dev()
    bits, scores = ck.cocktail_chunk_bitwidths(torch.from_numpy(q).to(dev), torch.from_numpy(np.concatenate(cs)).to(dev),
                                               num_chunks, alpha, beta)
    torch.cuda.synchronize()
    bits, scores = bits.cpu().numpy(), scores.cpu().numpy()
    pos = 0
    for b, n in enumerate(num_chunks):
        rb, rs = O.chunk_bitwidths(q[b], cs[b], alpha, beta)
        assert np.array_equal(scores[pos:pos + n], rs), f"scores of sequence {b} differ"
        assert np.array_equal(bits[pos:pos + n], rb), f"bitwidths of sequence {b} differ"
        pos += n
    # the result feeds the planner directly
    shape = ck.make_shape(len(num_chunks), 2, 2, 128, 32, 32)
    plan = ck.cocktail_plan(shape, [32 * n for n in num_chunks], bits, 64)
    assert int(plan.sizes.total_chunks) == sum(num_chunks)


def test_many_calls_with_changing_ticket_order_all_agree():
    """The hand-out order of the pool pieces changes from call to call; every call must still read each
    token exactly once.  200 calls on a pooled shape against the oracle's answer."""
    w = workloads.small("soak", 2, 4, 4, [9000, 5000], 128, 32, mix=(0.15, 0.35, 0.5), seed_offset=91)
    _announce(w.name)
    c = Case(w, workers=40)
    assert _counters(c)[1] > 0
    c.check_all()
    ref = c.out_dev.float()
    scale = ref.abs().amax(dim=2, keepdim=True)
    worst = 0.0
    for i in range(200):
        out, _ = ck.cocktail_decode_attention(c.cache, c.q_dev)
        err = ((out.float() - ref).abs() / scale).max().item()
        worst = max(worst, err)
        assert err <= 1e-3, f"call {i}: deviates from the first call by {err:.3e}"
    torch.cuda.synchronize()
    assert (_counters(c)[0] == 0).all()
    _announce(f"{w.name}: largest deviation between calls {worst:.2e}")


@pytest.mark.parametrize("rep", [1, 4, 8])
def test_reproducible_plan_gives_bitwise_identical_results(rep):
    w = workloads.small(f"repro_r{rep}", 2, 2 * rep, 2, [6000, 3000], 64, 64, mix=(0.2, 0.4, 0.4), seed_offset=88)
    _announce(w.name)
    dev = _dev()
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = np.concatenate(workloads.chunk_bits(w))
    k, v = workloads.kv_flat(w, 0)
    k_dev, v_dev = torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev)
    q_dev = torch.from_numpy(workloads.query(w, 0)).to(dev)
    outs = []
    for reproducible in (True, False):
        plan = ck.cocktail_plan(shape, w.seq_lens, bits, 8, reproducible=reproducible)
        cache = ck.PackedCache(plan, dev)
        ck.cocktail_reorder_quantize(cache, k_dev, v_dev, ragged=True)
        runs = [ck.cocktail_decode_attention(cache, q_dev)[0].clone() for _ in range(4)]
        torch.cuda.synchronize()
        if reproducible:
            assert all(torch.equal(runs[0], r) for r in runs[1:])
        outs.append(runs[0].float())
    # both splits compute the same attention
    assert (outs[0] - outs[1]).abs().max() <= 2e-3 * outs[0].abs().max()


def test_quantizer_division_shortcuts_are_exact_on_every_operand():
    """The kernel's replacements for (mx - mn) / qmax and 1 / scale against the IEEE divisions, exhaustively."""
    assert ck.cocktail_selftest_arithmetic(_dev()) == [0, 0, 0, 0]


def test_marked_call_equals_the_plain_call_and_records_its_event():
    """cocktail_decode_attention_marked (a measurement aid) computes what cocktail_decode_attention computes and
    records the caller's event between the two kernels."""
    w = workloads.small("marked", 2, 8, 2, [700, 64 * 6], 32, 32, mix=(0.2, 0.4, 0.4), seed_offset=77)
    _announce(w.name)
    c = Case(w, workers=16)
    out = torch.empty_like(c.out_dev)
    lse = torch.empty_like(c.lse_dev)
    start, mid, end = (torch.cuda.Event(enable_timing=True) for _ in range(3))
    mid.record()                                           # creates the handle
    torch.cuda.synchronize()
    start.record()
    ck.cocktail_decode_attention_marked(c.cache, c.q_dev, mid, out, lse)
    end.record()
    torch.cuda.synchronize()
    ck.cocktail_decode_check(c.cache)
    assert start.elapsed_time(mid) > 0 and mid.elapsed_time(end) > 0
    got = out.cpu().numpy().astype(np.float64)
    ref = c.out.astype(np.float64)
    assert (np.abs(got - ref).max(axis=2) / np.abs(ref).max(axis=2)).max() <= 1e-3     # pool tickets may be drawn in another order
    from paper_2503_23294_amd import _lib
    import ctypes as C
    rc = _lib.lib().cocktail_decode_attention_marked(C.byref(c.shape), c.q_dev.data_ptr(), C.byref(c.cache.desc), 0.0, out.data_ptr(),
                                                     lse.data_ptr(), c.cache.workspace.data_ptr(), c.cache.workspace.numel(), None, None)
    assert rc == _lib.EINVAL


def test_runs_on_a_side_stream():
    w = workloads.small("stream", 1, 2, 2, [512], 64, 32, seed_offset=4)
    _announce(w.name)
    c = Case(w, workers=8)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        out, _ = ck.cocktail_decode_attention(c.cache, c.q_dev)
    s.synchronize()
    assert torch.equal(out, c.out_dev)


def test_rejects_bad_device_arguments():
    w = workloads.small("bad", 1, 2, 2, [128], 64, 32)
    c = Case(w, workers=2)
    with pytest.raises(TypeError):
        ck.cocktail_decode_attention(c.cache, c.q_dev.float())
    small_ws = c.cache.workspace
    c.cache.workspace = small_ws[:16]
    with pytest.raises(ck.CocktailError) as e:
        ck.cocktail_decode_attention(c.cache, c.q_dev)
    assert e.value.code == -4
    c.cache.workspace = small_ws


def test_stream_read_probe_reads_what_it_reports_and_rejects_small_buffers():
    dev = torch.device("cuda:0")
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    buf = torch.zeros((48 << 20) + 4096, dtype=torch.uint8, device=dev)
    assert ck.cocktail_stream_read_probe(buf, sink) == 48 << 20     # rounded down to 2048 waves x 8 KiB
    torch.cuda.synchronize()
    assert int(sink.item()) == 0                                    # zeros never match the sentinel
    with pytest.raises(ck.CocktailError) as e:
        ck.cocktail_stream_read_probe(buf[:1 << 20], sink)
    assert e.value.code == -1
    with pytest.raises(ck.CocktailError) as e:
        ck.cocktail_stream_read_probe(buf[8:], sink)
    assert e.value.code == -3


@pytest.mark.parametrize("chunk", [8, 16, 32, 64, 128, 256])
def test_chunk_sizes_of_the_papers_sweep(chunk):
    """The chunk sizes the paper sweeps (Table III); 32 is its default."""
    w = workloads.small(f"chunk{chunk}", 2, 4, 4, [2048 + 3 * chunk + 5, 1024 + chunk // 2], chunk, 32,
                        mix=(0.1, 0.3, 0.6), seed_offset=300 + chunk)
    _announce(w.name)
    Case(w, workers=24).check_all()


def test_one_million_token_context():
    """A single very long sequence: block offsets inside one (sequence, head, class) run reach hundreds of
    megabytes, and one head's partials come from every worker."""
    w = workloads.small("million", 1, 2, 1, [(1 << 20) + 37], 1024, 64, mix=(0.3, 0.3, 0.4), seed_offset=123)
    _announce(w.name)
    c = Case(w)
    worst = c.check_all()
    _announce(f"{w.name} worst rel err {worst:.2e}")


# ---- full-size configurations, launch configuration of the bench, sampled heads ----------------
def _sample_heads(w, n, seed):
    rng = np.random.default_rng(seed)
    allh = [(b, h) for b in range(w.batch) for h in range(w.num_kv_heads)]
    pick = rng.choice(len(allh), size=min(n, len(allh)), replace=False)
    return sorted(allh[i] for i in pick)


@pytest.mark.parametrize("layer", [0, 15, 31])
def test_config2_layers(layer):
    w = workloads.config(2)
    _announce(f"config 2 layer {layer}")
    c = Case(w, layer=layer)
    c.check_plan()
    for b, h in _sample_heads(w, 4, layer):
        _announce(f"  head {b},{h}: {c.check_head(b, h):.2e}")


def test_config3_gqa_batch4():
    w = workloads.config(3)
    _announce("config 3")
    c = Case(w)
    c.check_plan()
    for b, h in _sample_heads(w, 6, 3):
        _announce(f"  head {b},{h}: {c.check_head(b, h):.2e}")


def test_config4_128k():
    w = workloads.config(4)
    _announce("config 4")
    c = Case(w)
    c.check_plan()
    for b, h in _sample_heads(w, 8, 4):
        _announce(f"  head {b},{h}: {c.check_head(b, h):.2e}")


def test_config5_ragged_dirichlet():
    w = workloads.config(5)
    _announce(f"config 5 lens={w.seq_lens}")
    c = Case(w)
    c.check_plan()
    heads = sorted(set(_sample_heads(w, 6, 5) + [(0, 0), (1, 7)]))   # seq 0 all-FP16, seq 1 all-INT2
    for b, h in heads:
        _announce(f"  head {b},{h}: {c.check_head(b, h):.2e}")


@pytest.mark.parametrize("rep", [1, 4, 8])
@pytest.mark.parametrize("kscale,vscale,qscale", [(1.0, 2.0e4, 1.0), (1.0, 1.0e-3, 1.0), (6.0, 1.0, 1.0), (0.02, 3.0e-3, 1.0),
                                                  (3.0, 5.0e-5, 1.0), (1.0, 2.0e4, 0.01), (1.0, 1.0, 1.0e-3), (0.1, 6.0e3, 0.05)])
def test_value_ranges_from_tiny_to_near_the_fp16_limit(rep, kscale, vscale, qscale):
    """V from fp16-subnormal magnitudes to values near 65504, peaked and flat softmax (a small query makes every
    token weigh the same, so the roundings of the weights that the matrix kernel feeds to its instructions in
    fp16 add up over all tokens instead of a few): same tolerance."""
    w = workloads.small(f"range_r{rep}", 2, 2 * rep, 2, [64 * 7 + 9, 64 * 3], 64, 32, mix=(0.2, 0.4, 0.4),
                        seed_offset=300 + rep)
    _announce(f"{w.name} k x{kscale} v x{vscale} q x{qscale}")
    dev = _dev()
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = workloads.chunk_bits(w)
    ks, vs = [], []
    for b in range(w.batch):
        kh, vh = zip(*[workloads.kv_head(w, 0, b, h) for h in range(w.num_kv_heads)])
        ks.append(np.clip(np.stack(kh).astype(np.float32) * kscale, -6.0e4, 6.0e4).astype(np.float16))
        vs.append(np.clip(np.stack(vh).astype(np.float32) * vscale, -6.0e4, 6.0e4).astype(np.float16))
    plan = ck.cocktail_plan(shape, w.seq_lens, np.concatenate(bits), 6)
    cache = ck.PackedCache(plan, dev)
    k_flat = np.concatenate([x.reshape(-1, w.head_dim) for x in ks])      # ragged: per sequence [Hkv][T_b] rows
    v_flat = np.concatenate([x.reshape(-1, w.head_dim) for x in vs])
    ck.cocktail_reorder_quantize(cache, torch.from_numpy(k_flat).to(dev), torch.from_numpy(v_flat).to(dev), ragged=True)
    q = (workloads.query(w, 0).astype(np.float32) * qscale).astype(np.float16)
    out, lse = ck.cocktail_decode_attention(cache, torch.from_numpy(q).to(dev))
    torch.cuda.synchronize()
    oc = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    v_quads = int(plan.sizes.v_layout) == 1
    for c in range(O.NUM_CLASSES):
        assert np.array_equal(cache.k[c].cpu().numpy(), O.pack_class_buffer(oc, c, "k"))
        assert np.array_equal(cache.v[c].cpu().numpy(), O.pack_class_buffer(oc, c, "v", v_quads=v_quads))
    ref, rl = O.decode_attention(q, oc)
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max(axis=2) / np.abs(ref).max(axis=2)
    _announce(f"  max rel err {err.max():.2e}")
    assert err.max() <= TOL, f"max rel err {err.max():.3e}"
    assert np.abs(lse.cpu().numpy() - rl).max() <= 1e-4 * max(1.0, np.abs(rl).max())


@pytest.mark.parametrize("rep", [1, 4])
def test_decode_calls_replayed_from_a_captured_graph(rep):
    """The decode entry point only enqueues kernels (no memset, no allocation), so a caller can capture a
    run of calls in a HIP graph; every replay must give the eager result (and leave the counters at zero)."""
    w = workloads.small(f"graph_r{rep}", 2, 2 * rep, 2, [3000, 1700], 64, 32, mix=(0.2, 0.4, 0.4), seed_offset=500 + rep)
    _announce(w.name)
    c = Case(w, workers=16)
    c.check_all()
    eager = c.out_dev.clone()
    outs = [torch.empty_like(c.out_dev) for _ in range(3)]
    lses = [torch.empty_like(c.lse_dev) for _ in range(3)]

    def calls():
        for o, l in zip(outs, lses):
            ck.cocktail_decode_attention(c.cache, c.q_dev, c.sm_scale, out=o, lse=l)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls()                                   # warm-up outside the capture, as graph capture asks for
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
    for replay in range(4):
        for o in outs:
            o.zero_()
        ck.cocktail_decode_attention(c.cache, c.q_dev, c.sm_scale)   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert (_counters(c)[0] == 0).all()
        for o in outs:
            assert torch.allclose(o.float(), eager.float(), rtol=0, atol=2e-3 * float(eager.float().abs().max())), \
                f"replay {replay} differs from the eager result"


@pytest.mark.parametrize("rep", [1, 4])
def test_quantizer_corner_groups_are_bit_exact(rep):
    """Groups of signed zeros, a zero maximum over negative values, fp16 subnormals, the largest range:
    the packed bytes still equal the oracle's (whose definition takes a zero extreme as +0)."""
    w = workloads.small(f"corners_r{rep}", 1, 2 * rep, 2, [64 * 4 + 20], 64, 32, mix=(0.0, 0.5, 0.5), seed_offset=700 + rep)
    _announce(w.name)
    dev = _dev()
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = workloads.chunk_bits(w)
    ks, vs = [], []
    rng = np.random.default_rng(701)
    for b in range(w.batch):
        kh, vh = zip(*[workloads.kv_head(w, 0, b, h) for h in range(w.num_kv_heads)])
        k, v = np.stack(kh).copy(), np.stack(vh).copy()
        for x in (k, v):
            t = x.shape[1]
            x[:, 0:t:7, 0:32] = np.float16(0.0)                                  # all +0
            x[:, 1:t:7, 0:32] = np.float16(-0.0)                                 # all -0
            x[:, 2:t:7, 32:64] = np.where(rng.random(32) < 0.5, np.float16(0.0), np.float16(-0.0))   # mixed zeros
            x[:, 3:t:7, 64:96] = -np.abs(x[:, 3:t:7, 64:96])                     # negative values ...
            x[:, 3:t:7, 70] = np.float16(-0.0)                                   # ... with a zero maximum
            x[:, 4:t:7, 96:128] = (rng.integers(-40, 40, size=32) * 2.0 ** -24).astype(np.float16)   # subnormals
            x[:, 5:t:7, 0] = np.float16(65504.0)
            x[:, 5:t:7, 1] = np.float16(-65504.0)                                # the largest range
        ks.append(k), vs.append(v)
    plan = ck.cocktail_plan(shape, w.seq_lens, np.concatenate(bits), 4)
    cache = ck.PackedCache(plan, dev)
    k_flat = np.concatenate([x.reshape(-1, w.head_dim) for x in ks])
    v_flat = np.concatenate([x.reshape(-1, w.head_dim) for x in vs])
    ck.cocktail_reorder_quantize(cache, torch.from_numpy(k_flat).to(dev), torch.from_numpy(v_flat).to(dev), ragged=True)
    torch.cuda.synchronize()
    oc = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    v_quads = int(plan.sizes.v_layout) == 1
    for c in range(O.NUM_CLASSES):
        assert np.array_equal(cache.k[c].cpu().numpy(), O.pack_class_buffer(oc, c, "k")), f"K class {c}"
        assert np.array_equal(cache.v[c].cpu().numpy(), O.pack_class_buffer(oc, c, "v", v_quads=v_quads)), f"V class {c}"


def _random_case(seed):
    """A random small workload: any supported head ratio, group size, chunk size, batch, lengths, mix, workers."""
    rng = np.random.default_rng(9000 + seed)
    rep = int(rng.choice([1, 1, 2, 3, 4, 4, 5, 6, 8, 12, 16]))
    hkv = int(rng.integers(1, 4))
    batch = int(rng.integers(1, 5))
    head_dim = int(rng.choice([64, 128, 128]))
    group = int(rng.choice([32, 64, 128] if head_dim == 128 else [32, 64]))
    chunk = int(rng.choice([8, 32, 64, 100, 256]))
    lens = [int(x) for x in rng.integers(0, 2500, size=batch)]
    if rng.random() < 0.3:
        lens[int(rng.integers(0, batch))] = int(rng.integers(0, chunk))      # a tail-only (or empty) sequence
    mix = rng.dirichlet([1.0, 1.0, 1.0, 1.0])                                 # FP16, INT8, INT4, INT2
    if rng.random() < 0.25:
        mix = np.eye(4)[int(rng.integers(0, 4))]                              # a single class
    elif rng.random() < 0.3:
        mix[int(rng.integers(0, 4))] = 0.0                                    # an empty class
    workers = int(rng.choice([1, 2, 5, 8, 16, 33, 64, 200]))
    w = workloads.small(f"fuzz{seed}", batch, hkv * rep, hkv, lens, chunk, group, mix=tuple(float(x) for x in mix),
                        head_dim=head_dim, seed_offset=9000 + seed)
    return w, workers


@pytest.mark.parametrize("seed", range(32))
def test_random_shapes(seed):
    w, workers = _random_case(seed)
    _announce(f"{w.name}: B={w.batch} Hq={w.num_q_heads} Hkv={w.num_kv_heads} D={w.head_dim} G={w.group_size} C={w.chunk_size} "
              f"T={list(w.seq_lens)} mix={[round(m, 2) for m in w.mix]} workers={workers}")
    Case(w, workers=workers).check_all()
