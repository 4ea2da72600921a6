"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the mistake it would catch.  None of these compares the oracle with
a retyped copy of its own formula: the references are textbook attention written
five lines long on the raw inputs, torch's CPU scaled_dot_product_attention, an
exact-rational scalar brute force, closed forms and invariants.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import workloads
from oracle import brute
from oracle import cocktail_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _seqs(w, layer=0):
    ks, vs = [], []
    for b in range(w.batch):
        kh, vh = zip(*[workloads.kv_head(w, layer, b, h) for h in range(w.num_kv_heads)])
        ks.append(np.stack(kh))
        vs.append(np.stack(vh))
    return ks, vs


def _textbook(q, k, v, sm_scale):
    s = (k.astype(np.float64) @ q.astype(np.float64)) * sm_scale
    p = np.exp(s - s.max())
    p /= p.sum()
    return p @ v.astype(np.float64), np.log(np.exp(s - s.max()).sum()) + s.max()


# -- 1. all-FP16 is exact attention (Alg. 1 with only the mm branch) ------------------------
def test_all_fp16_equals_textbook_attention():
    w = workloads.small("allfp16", 2, 4, 2, [96, 77], 16, 32, mix=(1.0, 0.0, 0.0))
    ks, vs = _seqs(w)
    bits = workloads.chunk_bits(w)
    assert all((b == 16).all() for b in bits)
    cache = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    q = workloads.query(w, 0)
    out, lse = O.decode_attention(q, cache)
    for b in range(w.batch):
        for h in range(w.num_q_heads):
            ref, rl = _textbook(q[b, h], ks[b][h // 2], vs[b][h // 2], 1 / np.sqrt(128))
            np.testing.assert_allclose(out[b, h], ref, rtol=0, atol=1e-12)
            assert abs(lse[b, h] - rl) < 1e-12


def test_all_fp16_equals_torch_sdpa():
    w = workloads.small("sdpa", 1, 4, 4, [200], 8, 32, mix=(1.0, 0.0, 0.0))
    ks, vs = _seqs(w)
    cache = O.reorder_quantize(ks, vs, workloads.chunk_bits(w), w.chunk_size, w.group_size)
    q = workloads.query(w, 0)
    out, _ = O.decode_attention(q, cache)
    tq = torch.from_numpy(q.astype(np.float32))[0][:, None, :]            # [H, 1, D]
    tk = torch.from_numpy(ks[0].astype(np.float32))
    tv = torch.from_numpy(vs[0].astype(np.float32))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, 0].numpy()
    np.testing.assert_allclose(out[0], ref, rtol=0, atol=1e-5)


# -- 2. permutation invariance (Sec. III-C, Eq. 4-5) ---------------------------------------
def test_reordering_does_not_change_output():
    w = workloads.small("perm", 1, 2, 2, [16 * 12 + 5], 16, 32, mix=(0.3, 0.3, 0.4))
    ks, vs = _seqs(w)
    bits = workloads.chunk_bits(w)
    assert len(set(bits[0].tolist())) == 3
    cache = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    q = workloads.query(w, 0)
    out, lse = O.decode_attention(q, cache)
    # same quantiser applied chunk by chunk with the cache left in ORIGINAL token order
    t, c = w.seq_lens[0], w.chunk_size
    for h in range(2):
        kh = np.empty((t, 128))
        vh = np.empty((t, 128))
        for i, b in enumerate(bits[0]):
            sl = slice(i * c, (i + 1) * c)
            if b == 16:
                kh[sl], vh[sl] = ks[0][h, sl], vs[0][h, sl]
            else:
                kh[sl] = O.dequantize(*O.quantize_rows(ks[0][h, sl], int(b), 32), 32)
                vh[sl] = O.dequantize(*O.quantize_rows(vs[0][h, sl], int(b), 32), 32)
        kh[(t // c) * c:], vh[(t // c) * c:] = ks[0][h, (t // c) * c:], vs[0][h, (t // c) * c:]
        ref, rl = _textbook(q[0, h], kh, vh, 1 / np.sqrt(128))
        np.testing.assert_allclose(out[0, h], ref, rtol=0, atol=1e-12)
        assert abs(lse[0, h] - rl) < 1e-12


def test_plan_is_stable_partition_and_tail_is_fp16():
    bits = np.array([4, 2, 16, 2, 4, 4, 16, 2], dtype=np.uint8)
    sp = O.plan_sequence(8 * 8 + 3, 8, bits)
    assert sp.perm.tolist() == [1, 3, 7, 0, 4, 5, 2, 6]          # INT2 | INT4 | FP16, each ascending
    assert sp.class_tokens == (24, 24, 0, 16 + 3) and sp.tail == 3
    idx = O.class_token_index(67, 8, sp)
    assert idx[O.FP16_CLASS].tolist()[-3:] == [64, 65, 66]         # tail follows the FP16 chunks
    assert sorted(np.concatenate(idx).tolist()) == list(range(67))
    # with INT8 chunks: INT2 | INT4 | INT8 | FP16, by precision
    bits = np.array([8, 16, 2, 8, 4, 2], dtype=np.uint8)
    sp = O.plan_sequence(6 * 4 + 1, 4, bits)
    assert sp.perm.tolist() == [2, 5, 4, 0, 3, 1] and sp.class_tokens == (8, 4, 8, 4 + 1)
    assert O.class_token_index(25, 4, sp)[2].tolist() == [0, 1, 2, 3, 12, 13, 14, 15]


# -- 3. quantisation bound and extremes ----------------------------------------------------
@pytest.mark.parametrize("bits,group", [(2, 32), (4, 32), (2, 64), (4, 64), (2, 128), (4, 128), (8, 32), (8, 64), (8, 128)])
def test_quantisation_error_at_most_half_a_step(bits, group):
    rng = np.random.default_rng(7)
    x = rng.standard_normal((512, 128)).astype(np.float32)
    x[:, [3, 40, 77, 100]] *= 10
    x = x.astype(np.float16)
    codes, scale, zero = O.quantize_rows(x, bits, group)
    qmax = (1 << bits) - 1
    assert codes.min() >= 0 and codes.max() <= qmax
    xh = O.dequantize(codes, scale, zero, group)
    sc = np.repeat(scale.astype(np.float64), group, axis=-1)
    # half a step, plus what the fp16 rounding of the scale (relative 2^-11) can add at the far end of the
    # range: up to qmax * 2^-11 steps, which only shows at 8 bits
    assert (np.abs(x.astype(np.float64) - xh) <= (0.5 * (1 + 1e-4) + qmax * 2.0 ** -11) * sc + 1e-30).all()
    cg = codes.reshape(512, 128 // group, group)
    assert (cg.min(-1) == 0).all() and (cg.max(-1) == qmax).all()   # min -> 0, max -> qmax
    xg = x.reshape(512, 128 // group, group)
    assert (zero == xg.min(-1)).all()


def test_closed_form_groups():
    row = np.tile(np.arange(4, dtype=np.float16), 32)[None]                   # {0,1,2,3}: scale 1, zero 0
    c, s, z = O.quantize_rows(row, 2, 32)
    assert (c == row).all() and (s == 1).all() and (z == 0).all()
    row = np.tile(np.arange(16, dtype=np.float16), 8)[None]
    c, s, z = O.quantize_rows(row, 4, 64)
    assert (c == row).all() and (s == 1).all() and (z == 0).all()
    # 8 bits: integers of [0, 255] with 0 and 255 in every group: scale 1, zero 0, codes = values
    grp = np.array([0, 255] + [17, 200, 3, 128] * 7 + [9, 77], dtype=np.float16)
    c, s, z = O.quantize_rows(np.tile(grp, 4)[None], 8, 32)
    assert (s == 1).all() and (z == 0).all() and (c == np.tile(grp, 4)[None]).all()
    row = np.array([0, 255] + list(range(1, 127)), dtype=np.float16)[None]          # one group of 128 channels
    c, s, z = O.quantize_rows(row, 8, 128)
    assert (c == row).all() and (s == 1).all() and (z == 0).all()
    const = np.full((1, 128), -2.5, dtype=np.float16)                          # constant: scale 0, exact
    c, s, z = O.quantize_rows(const, 4, 32)
    assert (c == 0).all() and (s == 0).all() and (z == np.float16(-2.5)).all()
    assert (O.dequantize(c, s, z, 32) == -2.5).all()
    # affine ramp a + k*h with qmax steps is reproduced exactly
    ramp = (np.float16(-3.0) + np.float16(0.5) * np.arange(16)).astype(np.float16)
    c, s, z = O.quantize_rows(np.tile(ramp, 8)[None], 4, 32)
    assert (c == np.tile(np.arange(16), 8)).all() and (s == 0.5).all() and (z == -3).all()
    # ties go to even: x - mn = 0.5, 1.5, 2.5 steps
    x = np.array([0, 3, 0.5, 1.5, 2.5] + [0] * 27, dtype=np.float16)
    c, _, _ = O.quantize_rows(x[None], 2, 32)
    assert c[0, :5].tolist() == [0, 3, 0, 2, 2]


def test_two_equal_logits_and_dominant_token():
    d = 128
    k = np.zeros((1, 2, d), dtype=np.float16)
    v = np.stack([np.full(d, 1.0), np.full(d, 3.0)]).astype(np.float16)[None]
    cache = O.reorder_quantize([k], [v], [np.zeros(0, np.uint8)], 8, 32)       # both tokens are tail
    q = np.ones((1, 1, d), dtype=np.float16)
    out, lse = O.decode_attention(q, cache)
    np.testing.assert_allclose(out[0, 0], 2.0, atol=1e-15)
    assert abs(lse[0, 0] - np.log(2)) < 1e-15
    k[0, 1, 0] = 60 * np.sqrt(d)                                                # logit +60
    cache = O.reorder_quantize([k], [v], [np.zeros(0, np.uint8)], 8, 32)
    out, _ = O.decode_attention(q, cache)
    np.testing.assert_allclose(out[0, 0], 3.0, atol=1e-20 + 3 * np.exp(-59.0))


# -- 4. exact-rational brute force on tiny inputs ------------------------------------------
def test_rounding_helper_matches_ieee():
    from fractions import Fraction
    rng = np.random.default_rng(0)
    for v in rng.standard_normal(200) * 10.0 ** rng.integers(-9, 5, 200):
        fr = Fraction(float(v))
        assert float(brute.rn32(fr)) == float(np.float32(v))
        if abs(v) < 6e4:
            assert float(brute.rn16(fr)) == float(np.float16(v))
    assert brute.rn16(Fraction(2049)) == 2048 and brute.rn16(Fraction(2051)) == 2052   # ties to even
    assert brute.rn16(Fraction(1, 2 ** 25)) == 0 and brute.rn16(Fraction(3, 2 ** 25)) == Fraction(1, 2 ** 23)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantiser_matches_exact_rational_brute_force(bits):
    rng = np.random.default_rng(11 + bits)
    x = rng.standard_normal((40, 64)).astype(np.float32)
    x[:, 5] *= 10
    x[7] *= 1e-4                       # small magnitudes: fp16 subnormal scales
    x[8] = 0.125                       # constant
    x[9, :3] = [0.0, -0.0, 1e-7]
    x = x.astype(np.float16)
    for group in (32, 64):
        codes, scale, zero = O.quantize_rows(x, bits, group)
        for t in range(x.shape[0]):
            for g in range(64 // group):
                bc, bs, bz = brute.quantize_group([float(v) for v in x[t, g * group:(g + 1) * group]], bits)
                assert bc == codes[t, g * group:(g + 1) * group].tolist(), (t, g)
                assert bs == float(scale[t, g]) and bz == float(zero[t, g])
                assert not np.signbit(zero[t, g]) or zero[t, g] != 0


def _tiny_case(bsz, hkv, rep, d, t_list, chunk, group, assign, seed):
    rng = np.random.default_rng(seed)
    ks = [rng.standard_normal((hkv, t, d)).astype(np.float16) for t in t_list]
    vs = [rng.standard_normal((hkv, t, d)).astype(np.float16) for t in t_list]
    q = rng.standard_normal((bsz, hkv * rep, d)).astype(np.float16)
    return ks, vs, q, [np.array(a, dtype=np.uint8) for a in assign]


@pytest.mark.parametrize("d,chunk,t", [(64, 4, 14), (64, 8, 27), (128, 5, 17)])
def test_full_path_matches_brute_force_all_assignments(d, chunk, t):
    n = t // chunk
    group = 32
    every = list(itertools.product((2, 4, 8, 16), repeat=n))
    if d > 64 or t > 20:
        every = every[::5]             # the scalar brute force is slow: all 4^n assignments for the smallest case only
    for assign in every:
        ks, vs, q, bits = _tiny_case(1, 2, 2, d, [t], chunk, group, [assign], seed=hash(assign) % 1000)
        cache = O.reorder_quantize(ks, vs, bits, chunk, group)
        order, tok = brute.plan(t, chunk, list(assign))
        assert cache.plans[0].perm.tolist() == order
        assert list(cache.plans[0].class_tokens) == [len(x) for x in tok]
        kl = [[[float(x) for x in row] for row in ks[0][h]] for h in range(2)]
        vl = [[[float(x) for x in row] for row in vs[0][h]] for h in range(2)]
        for cls, b in enumerate((2, 4, 8, 16)):
            assert O.pack_class_buffer(cache, cls, "k").tobytes() == brute.build_class_bytes(kl, tok[cls], b, group)
            assert O.pack_class_buffer(cache, cls, "v").tobytes() == brute.build_class_bytes(vl, tok[cls], b, group)
        out, lse = O.decode_attention(q, cache, sm_scale=0.3)
        for hq in range(4):
            h = hq // 2
            krows = [brute.dequant_token(kl[h][tt], b, group) for b, ts in zip((2, 4, 8, 16), tok) for tt in ts]
            vrows = [brute.dequant_token(vl[h][tt], b, group) for b, ts in zip((2, 4, 8, 16), tok) for tt in ts]
            bo, bl = brute.attention([float(x) for x in q[0, hq]], krows, vrows, 0.3)
            np.testing.assert_allclose(out[0, hq], bo, rtol=0, atol=1e-12)
            assert abs(lse[0, hq] - bl) < 1e-12


def test_ragged_batch_brute_force_block_tail():
    # 70 INT2 tokens -> two 64-token blocks, the second with 6 valid tokens; sequences of different length
    ks, vs, q, bits = _tiny_case(2, 1, 1, 64, [70, 9], 70, 32, [[2], []], seed=3)
    bits[1] = np.zeros(0, dtype=np.uint8)
    cache = O.reorder_quantize(ks, vs, bits, 70, 32)
    kl = [[[float(x) for x in row] for row in ks[0][0]]]
    _, tok = brute.plan(70, 70, [2])
    buf = O.pack_class_buffer(cache, 0, "k")
    assert buf.size == 2 * O.block_bytes(0, 64, 32)
    assert buf.tobytes() == brute.build_class_bytes(kl, tok[0], 2, 32)
    # second sequence: 9 tail tokens only, FP16 class
    assert cache.plans[1].class_tokens == (0, 0, 0, 9)
    fp = O.pack_class_buffer(cache, O.FP16_CLASS, "k")
    kl1 = [[[float(x) for x in row] for row in ks[1][0]]]
    assert fp.tobytes() == brute.build_class_bytes(kl1, list(range(9)), 16, 32)


# -- 5. pack / unpack round trip and byte count ---------------------------------------------
def test_pack_round_trip_and_sizes():
    w = workloads.small("rt", 2, 2, 2, [64 * 3 + 40, 200], 8, 32, mix=(0.2, 0.2, 0.2, 0.4))
    ks, vs = _seqs(w)
    cache = O.reorder_quantize(ks, vs, workloads.chunk_bits(w), 8, 32)
    assert all(cache.seqs[0][c].n_tokens > 0 for c in range(O.NUM_CLASSES))
    for cls in range(O.NUM_CLASSES):
        for which in "kv":
            buf = O.pack_class_buffer(cache, cls, which)
            nblk = sum(((s[cls].n_tokens + 63) // 64) * 2 for s in cache.seqs)
            assert buf.size == nblk * O.block_bytes(cls, 128, 32)
            back = O.unpack_class_buffer(buf, cache, cls)
            for b in range(2):
                cc = cache.seqs[b][cls]
                if cc.n_tokens == 0:
                    continue
                for h in range(2):
                    if cls == O.FP16_CLASS:
                        ref = (cc.k_raw if which == "k" else cc.v_raw)[h]
                        assert (back[b][h][0] == ref).all()
                    else:
                        assert (back[b][h][0] == (cc.k_codes if which == "k" else cc.v_codes)[h]).all()
                        assert (back[b][h][1] == (cc.k_scale if which == "k" else cc.v_scale)[h]).all()
                        assert (back[b][h][2] == (cc.k_zero if which == "k" else cc.v_zero)[h]).all()
    # algorithmic bytes: 48 / 80 / 144 / 256 per (token, head) at G=32
    assert O.packed_bytes((1, 0, 0, 0), 1, 128, 32) == 2 * 48
    assert O.packed_bytes((0, 1, 0, 0), 1, 128, 32) == 2 * 80
    assert O.packed_bytes((0, 0, 1, 0), 1, 128, 32) == 2 * 144
    assert O.packed_bytes((0, 0, 0, 1), 1, 128, 64) == 2 * 256
    assert O.packed_bytes((1, 1, 0, 0), 1, 128, 64) == 2 * (40 + 72)
    assert O.packed_bytes((1, 1, 1, 1), 1, 64, 32) == 2 * (24 + 40 + 72 + 128)


def test_row_word_layout_by_hand():
    codes = np.zeros(128, dtype=np.uint8)
    codes[0], codes[1], codes[2], codes[15], codes[16] = 1, 2, 3, 3, 2
    w = O.pack_row_words(codes, 2)
    assert w.shape == (8,)
    # ch0 -> bit 0, ch1 -> bit 16, ch2 -> bit 2, ch15 -> bits 30..31, ch16 -> word 1 bit 0
    assert int(w[0]) == (1 << 0) | (2 << 16) | (3 << 2) | (3 << 30) and int(w[1]) == 2
    codes = np.zeros(128, dtype=np.uint8)
    codes[0], codes[1], codes[6], codes[7], codes[8] = 15, 1, 9, 5, 7
    w = O.pack_row_words(codes, 4)
    assert int(w[0]) == 15 | (1 << 16) | (9 << 12) | (5 << 28) and int(w[1]) == 7
    assert (O.unpack_row_words(w, 4) == codes).all()
    # 8 bits: four channels per word, ch0 -> bits 0..7, ch1 -> bits 16..23, ch2 -> bits 8..15, ch3 -> bits 24..31
    codes = np.zeros(64, dtype=np.uint8)
    codes[0], codes[1], codes[2], codes[3], codes[4] = 0xA1, 0xB2, 0xC3, 0xD4, 0x7F
    w = O.pack_row_words(codes, 8)
    assert w.shape == (16,) and int(w[0]) == 0xD4B2C3A1 and int(w[1]) == 0x7F
    assert (O.unpack_row_words(w, 8) == codes).all()


# -- 6. partial-softmax merge identity -------------------------------------------------------
def test_merging_partials_equals_global_softmax():
    rng = np.random.default_rng(5)
    s = rng.standard_normal(300) * 3
    v = rng.standard_normal((300, 16))
    p = np.exp(s - s.max())
    ref = (p / p.sum()) @ v
    cuts = [0, 0, 17, 17, 120, 300]                                    # includes empty splits
    ms, ls, os_ = [], [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        if a == b:
            ms.append(-np.inf), ls.append(0.0), os_.append(np.zeros(16))
            continue
        m = s[a:b].max()
        e = np.exp(s[a:b] - m)
        ms.append(m), ls.append(e.sum()), os_.append(e @ v[a:b])
    out, lse = O.merge_partials(ms, ls, os_)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)
    assert abs(lse - (np.log(p.sum()) + s.max())) < 1e-12
    assert O.merge_partials([], [], [])[0] is None


# -- 7. reorder and quantise commute; GQA = replicated MHA; ragged = separate calls ----------
def test_quantise_then_reorder_equals_reorder_then_quantise():
    w = workloads.small("comm", 1, 1, 1, [8 * 12], 8, 32, mix=(0.0, 0.3, 0.4, 0.3))
    ks, vs = _seqs(w)
    bits = workloads.chunk_bits(w)
    cache = O.reorder_quantize(ks, vs, bits, 8, 32)
    idx = O.class_token_index(96, 8, cache.plans[0])
    assert all(len(idx[c]) > 0 for c in range(3))
    for cls, b in ((0, 2), (1, 4), (2, 8)):
        c_all, s_all, z_all = O.quantize_rows(ks[0][0], b, 32)          # quantise in original order first
        assert (c_all[idx[cls]] == cache.seqs[0][cls].k_codes[0]).all()
        assert (s_all[idx[cls]] == cache.seqs[0][cls].k_scale[0]).all()
        assert (z_all[idx[cls]] == cache.seqs[0][cls].k_zero[0]).all()


def test_gqa_equals_replicated_mha_and_ragged_equals_single_calls():
    w = workloads.small("gqa", 2, 4, 2, [40, 88], 8, 32)
    ks, vs = _seqs(w)
    bits = workloads.chunk_bits(w)
    q = workloads.query(w, 0)
    out, lse = O.decode_attention(q, O.reorder_quantize(ks, vs, bits, 8, 32))
    for b in range(2):
        krep = [np.repeat(ks[b], 2, axis=0)]
        vrep = [np.repeat(vs[b], 2, axis=0)]
        o1, l1 = O.decode_attention(q[b:b + 1], O.reorder_quantize(krep, vrep, [bits[b]], 8, 32))
        np.testing.assert_array_equal(o1[0], out[b])
        np.testing.assert_array_equal(l1[0], lse[b])


def test_subset_of_heads_matches_full():
    w = workloads.small("subset", 1, 4, 2, [64], 8, 32)
    ks, vs = _seqs(w)
    cache = O.reorder_quantize(ks, vs, workloads.chunk_bits(w), 8, 32)
    q = workloads.query(w, 0)
    full, _ = O.decode_attention(q, cache)
    part, _ = O.decode_attention(q, cache, heads=[(0, 3)])
    np.testing.assert_array_equal(part[0, 3], full[0, 3])
    assert np.isnan(part[0, 0]).all()


# -- 8. the paper's KV-size figure (Sec. I) ---------------------------------------------------
def test_kv_size_figure_from_paper():
    with open(os.path.join(GOLDEN, "kv_cache_size_llama2_13b_128k.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    layers, heads, hd, tokens, gb, tol = rows[0]
    got = O.kv_bytes_fp16(int(layers), int(heads), int(hd), int(tokens)) / 1e9
    assert abs(got - float(gb)) / float(gb) <= float(tol)
    # the same count from the packed-bytes formula with every token in the FP16 class
    assert O.packed_bytes((0, 0, 0, int(tokens)), int(heads), int(hd), 64) * int(layers) / 1e9 == got


# -- appended decode tokens (Sec. III-A: generated tokens stay FP16 behind the context) --------
def _new_tokens(w, step):
    rng = np.random.default_rng([workloads.BASE_SEED, 991, step])
    shape = (w.batch, w.num_kv_heads, w.head_dim)
    return (rng.standard_normal(shape, dtype=np.float32).astype(np.float16),
            rng.standard_normal(shape, dtype=np.float32).astype(np.float16))


def test_appended_tokens_all_fp16_equal_textbook_attention_over_the_concatenation():
    w = workloads.small("app16", 2, 4, 2, [80, 33], 16, 32, mix=(1.0, 0.0, 0.0), seed_offset=21)
    ks, vs = _seqs(w)
    cache = O.reorder_quantize(ks, vs, workloads.chunk_bits(w), w.chunk_size, w.group_size)
    q = workloads.query(w, 0)
    for step in range(5):
        kn, vn = _new_tokens(w, step)
        O.append_tokens(cache, kn, vn)
        ks = [np.concatenate([k, kn[b][:, None, :]], axis=1) for b, k in enumerate(ks)]
        vs = [np.concatenate([v, vn[b][:, None, :]], axis=1) for b, v in enumerate(vs)]
        out, lse = O.decode_attention(q, cache)
        for b in range(w.batch):
            for h in range(w.num_q_heads):
                ref, rl = _textbook(q[b, h], ks[b][h // 2], vs[b][h // 2], 1 / np.sqrt(128))
                np.testing.assert_allclose(out[b, h], ref, rtol=0, atol=1e-12)
                assert abs(lse[b, h] - rl) < 1e-12


def test_appended_tokens_behave_like_the_fp16_remainder_of_a_longer_context():
    """T context tokens + n appended ones == a (T + n)-token context whose last n tokens do not fill a
    chunk and therefore stay FP16 (Sec. III-A), for the same chunk bitwidths."""
    t, n, chunk = 4 * 24, 7, 24
    w_long = workloads.small("applong", 1, 2, 2, [t + n], chunk, 32, mix=(0.2, 0.4, 0.4), seed_offset=23)
    ks, vs = _seqs(w_long)
    bits = workloads.chunk_bits(w_long)
    assert len(bits[0]) == t // chunk and len(set(bits[0].tolist())) >= 2
    long_cache = O.reorder_quantize(ks, vs, bits, chunk, 32)
    cache = O.reorder_quantize([ks[0][:, :t]], [vs[0][:, :t]], bits, chunk, 32)
    for i in range(n):
        O.append_tokens(cache, ks[0][None, :, t + i], vs[0][None, :, t + i])
    q = workloads.query(w_long, 0)
    a, la = O.decode_attention(q, cache)
    b_, lb = O.decode_attention(q, long_cache)
    np.testing.assert_allclose(a, b_, rtol=0, atol=1e-13)
    np.testing.assert_allclose(la, lb, rtol=0, atol=1e-13)
    # and the append buffer's byte image holds exactly those rows, in the FP16 block layout
    img = O.pack_append_buffer(cache, "k", 70)
    assert img.size == 2 * 2 * 64 * 256                      # 2 heads x 2 blocks
    blocks = img.reshape(2, 2, 64 * 256)
    for h in range(2):
        rows = blocks[h, 0].reshape(16, 64, 16).transpose(1, 0, 2).reshape(64, 256)
        assert np.array_equal(rows[:n], ks[0][h, t:t + n].view(np.uint8).reshape(n, 256))
        assert not rows[n:].any() and not blocks[h, 1].any()


# -- chunk-level quantization search (Sec. III-B, Eq. 1-3) --------------------------------------
def test_similarity_scores_equal_sklearn_cosine_and_closed_forms():
    from sklearn.metrics.pairwise import cosine_similarity
    q, cs = workloads.embeddings(5, [300, 1])
    s = O.similarity_scores(q[0], cs[0])
    ref = cosine_similarity(cs[0].astype(np.float64), q[0:1].astype(np.float64))[:, 0]
    assert s.dtype == np.float32
    np.testing.assert_allclose(s, ref, rtol=0, atol=6e-8)             # one float32 rounding
    e = np.eye(4, dtype=np.float32)
    c = np.stack([e[0], e[1], -e[0], 3 * e[0] + 4 * e[1], np.zeros(4, np.float32)])
    np.testing.assert_array_equal(O.similarity_scores(2 * e[0], c), np.float32([1, 0, -1, 0.6, 0]))
    # Eq. 1 does not depend on the lengths of the vectors (powers of two keep it bit for bit)
    np.testing.assert_array_equal(O.similarity_scores(4 * q[0], 0.5 * cs[0]), s)


def test_thresholds_worked_example_limits_and_order_of_comparisons():
    s = np.float32([0.1, 0.5, 0.9])
    t_low, t_high = O.thresholds(s, 0.6, 0.1)                        # Eq. 2: 0.1 + 0.8*0.6, Eq. 3: 0.9 - 0.8*0.1
    assert abs(t_low - 0.58) < 1e-6 and abs(t_high - 0.82) < 1e-6
    e = np.eye(3, dtype=np.float32)
    q = e[0]
    c = np.stack([0.1 * e[0] + np.sqrt(1 - 0.01) * e[1], 0.5 * e[0] + np.sqrt(0.75) * e[1],
                  0.9 * e[0] + np.sqrt(1 - 0.81) * e[1]]).astype(np.float32)
    bits, sc = O.chunk_bitwidths(q, c, 0.6, 0.1)
    np.testing.assert_allclose(sc, s, atol=1e-6)
    assert bits.tolist() == [2, 2, 16]
    # alpha = beta = 0: T_low = s_min, T_high = s_max, nothing lies strictly outside -> all INT4
    assert O.chunk_bitwidths(q, c, 0.0, 0.0)[0].tolist() == [4, 4, 4]
    # overlapping thresholds: the INT2 test comes first in Alg. 1's loop
    assert O.chunk_bitwidths(q, c, 0.9, 0.9)[0].tolist() == [2, 2, 16]
    # alpha = beta = 1: T_low = s_max, T_high = s_min; only the top chunk is not below T_low, and it is above T_high
    assert O.chunk_bitwidths(q, c, 1.0, 1.0)[0].tolist() == [2, 2, 16]
    # a single chunk, or equal scores: both thresholds equal the score -> INT4
    assert O.chunk_bitwidths(q, c[:1], 0.6, 0.1)[0].tolist() == [4]
    assert O.chunk_bitwidths(q, np.stack([c[1], c[1]]), 0.6, 0.1)[0].tolist() == [4, 4]
    assert O.chunk_bitwidths(q, c[:0], 0.6, 0.1)[0].size == 0


def test_more_alpha_means_more_int2_and_more_beta_means_more_fp16():
    """Sec. IV-C: a larger alpha sends more chunks to INT2, a larger beta keeps more in FP16."""
    q, cs = workloads.embeddings(6, [4096])
    prev2 = prev16 = -1
    for a in (0.0, 0.2, 0.4, 0.6, 0.8):
        bits, s = O.chunk_bitwidths(q[0], cs[0], a, 0.1)
        n2 = int((bits == 2).sum())
        assert n2 >= prev2
        prev2 = n2
        assert bits[np.argmax(s)] == 16 and (a == 0.0 or bits[np.argmin(s)] == 2)
    for b_ in (0.0, 0.1, 0.2, 0.3):
        bits, _ = O.chunk_bitwidths(q[0], cs[0], 0.6, b_)
        n16 = int((bits == 16).sum())
        assert n16 >= prev16
        prev16 = n16
    bits, _ = O.chunk_bitwidths(q[0], cs[0], 0.6, 0.1)                # the paper's defaults
    share = [(bits == v).mean() for v in (2, 4, 16)]
    assert share[0] > 0.5 and 0 < share[2] < 0.1                      # most chunks are irrelevant to the query


# -- token-quad form of V (grouped-query shapes) --------------------------------------------
def _quad_bytes_lane_by_lane(vals, bits, d):
    """The token-quad block image built the way a wave reads it: for every 32-token unit, lane,
    16-byte piece, word and half-word, which token and which channels end up there.  Pure loops."""
    n = vals.shape[0]
    nblk = (n + 63) // 64
    per = 16 // bits                       # values per half-word
    ph = (d * bits // 8) // 16 // (d // 64)  # pieces per lane (= per 64-channel half)
    out = bytearray(nblk * 64 * d * bits // 8)
    for blk in range(nblk):
        for u in range(2):
            for lane in range(64 * (d // 128) if d >= 128 else 32):
                t, h = lane % 32, lane // 32
                quad, j = t // 4, t % 4
                for word in range(4 * ph):
                    pair, tp = word // 2, word % 2
                    for hf in range(2):
                        tok = blk * 64 + 32 * u + 4 * quad + 2 * tp + hf
                        x = 0
                        for f in range(per):
                            e = pair * per + f
                            c = 64 * h + 32 * (e // 8) + 8 * j + e % 8
                            if tok < n:
                                x |= int(vals[tok, c]) << (f * bits)
                        addr = blk * (64 * d * bits // 8) + ((ph * h + word // 4) * 64 + 32 * u + t) * 16 + (word % 4) * 4 + 2 * hf
                        out[addr] = x & 0xff
                        out[addr + 1] = x >> 8
    return bytes(out)


@pytest.mark.parametrize("bits", [2, 4, 8, 16])
@pytest.mark.parametrize("d", [64, 128])
def test_token_quad_layout_matches_a_lane_by_lane_construction(bits, d):
    # catches: a wrong slot, word, half-word or bit position of the token-quad form; tokens past the end not zero
    rng = np.random.default_rng(bits * 10 + d)
    n = 64 + 37
    vals = rng.integers(0, 1 << bits, size=(n, d), dtype=np.uint32).astype(np.uint16)
    img = O.pack_quad_blocks(vals, bits, None)
    assert img.shape == (2, 64 * d * bits // 8)
    assert img.tobytes() == _quad_bytes_lane_by_lane(vals, bits, d)
    back, meta = O.unpack_quad_blocks(img, n, d, bits, 0)
    assert meta is None and (back == vals).all()


def test_token_quad_class_buffer_holds_the_same_values_and_meta():
    # catches: the quad form losing or reordering meta, touching K, or changing the block size
    w = workloads.small("quads", 2, 8, 2, [64 * 2 + 40, 130], 8, 32, mix=(0.2, 0.2, 0.2, 0.4))
    ks, vs = _seqs(w)
    cache = O.reorder_quantize(ks, vs, workloads.chunk_bits(w), 8, 32)
    for cls in range(O.NUM_CLASSES):
        assert O.pack_class_buffer(cache, cls, "k", v_quads=True).tobytes() == O.pack_class_buffer(cache, cls, "k").tobytes()
        rows = O.pack_class_buffer(cache, cls, "v")
        quads = O.pack_class_buffer(cache, cls, "v", v_quads=True)
        assert rows.size == quads.size
        bb = O.block_bytes(cls, 128, 32)
        bits = O.CLASS_BITS[cls]
        mb = 0 if cls == O.FP16_CLASS else 4 * 128 // 32
        pos = 0
        for b in range(2):
            cc = cache.seqs[b][cls]
            if cc.n_tokens == 0:
                continue
            nblk = (cc.n_tokens + 63) // 64
            for h in range(2):
                blk = quads[pos:pos + nblk * bb].reshape(nblk, bb)
                vals, meta = O.unpack_quad_blocks(blk, cc.n_tokens, 128, bits, mb)
                if cls == O.FP16_CLASS:
                    assert (vals == cc.v_raw[h].view(np.uint16)).all()
                else:
                    assert (vals == cc.v_codes[h]).all()
                    # meta bytes are those of the row form
                    assert (blk[:, 64 * 128 * bits // 8:] == rows[pos:pos + nblk * bb].reshape(nblk, bb)[:, 64 * 128 * bits // 8:]).all()
                    m = np.ascontiguousarray(meta).view("<f2").reshape(cc.n_tokens, 4, 2)
                    assert (m[..., 0] == cc.v_scale[h]).all() and (m[..., 1] == cc.v_zero[h]).all()
                pos += nblk * bb
        assert pos == quads.size


def test_token_quad_append_buffer():
    # catches: appended V rows not following the quad form; K rows changed
    w = workloads.small("quadapp", 1, 4, 1, [40], 8, 32, mix=(0.3, 0.3, 0.4))
    ks, vs = _seqs(w)
    cache = O.reorder_quantize(ks, vs, workloads.chunk_bits(w), 8, 32)
    rng = np.random.default_rng(5)
    for _ in range(3):
        O.append_tokens(cache, rng.standard_normal((1, 1, 128)).astype(np.float16), rng.standard_normal((1, 1, 128)).astype(np.float16))
    assert O.pack_append_buffer(cache, "k", 70, v_quads=True).tobytes() == O.pack_append_buffer(cache, "k", 70).tobytes()
    img = O.pack_append_buffer(cache, "v", 70, v_quads=True).reshape(2, -1)
    vals, _ = O.unpack_quad_blocks(img, 70, 128, 16, 0)
    assert (vals[:3] == cache.app_v[0][0].view(np.uint16)).all() and not vals[3:].any()


def test_signed_zeros_do_not_reach_scale_or_zero():
    # catches: the sign of a zero extreme leaking into the stored scale or zero (it would depend on element order)
    for order in ([-0.0, 0.0], [0.0, -0.0], [-0.0, -0.0], [0.0, 0.0]):
        x = np.array([order * 16], dtype=np.float16)
        for bits in (2, 4, 8):
            codes, scale, zero = O.quantize_rows(x, bits, 32)
            assert scale.view(np.uint16).item() == 0 and zero.view(np.uint16).item() == 0 and not codes.any()
    # a group whose maximum is a zero and whose minimum is negative: range = -min exactly, whatever the zero's sign
    for z in (0.0, -0.0):
        x = np.array([[-3.0, z] + [-1.5] * 30], dtype=np.float16)
        codes, scale, zero = O.quantize_rows(x, 2, 32)
        assert float(scale[0, 0]) == 1.0 and float(zero[0, 0]) == -3.0 and codes[0, :3].tolist() == [0, 3, 2]


def test_sequences_that_stop_generating_at_different_steps_equal_single_sequence_runs():
    # catches: a skipped sequence still receiving a row, rows of one sequence landing in another, a step miscounted
    w = workloads.small("raggedgen", 3, 4, 2, [70, 33, 120], 16, 32, mix=(0.2, 0.4, 0.4), seed_offset=29)
    ks, vs = _seqs(w)
    bits = workloads.chunk_bits(w)
    q = workloads.query(w, 0)
    cache = O.reorder_quantize(ks, vs, bits, w.chunk_size, w.group_size)
    singles = [O.reorder_quantize([ks[b]], [vs[b]], [bits[b]], w.chunk_size, w.group_size) for b in range(3)]
    stops = [2, 0, 5]                                     # sequence 1 generates nothing, 0 stops after 2 tokens
    for step in range(5):
        kn, vn = _new_tokens(w, 100 + step)
        active = [step < stops[b] for b in range(3)]
        O.append_tokens(cache, kn, vn, active)
        for b in range(3):
            if active[b]:
                O.append_tokens(singles[b], kn[b:b + 1], vn[b:b + 1])
    assert [cache.app_k[b].shape[1] for b in range(3)] == stops
    out, lse = O.decode_attention(q, cache)
    for b in range(3):
        o1, l1 = O.decode_attention(q[b:b + 1], singles[b])
        np.testing.assert_array_equal(out[b], o1[0])
        np.testing.assert_array_equal(lse[b], l1[0])
        # and the single-sequence run is textbook attention over context + its own appended rows (all-FP16 check is
        # test_appended_tokens_all_fp16_equal_textbook_attention_over_the_concatenation)
    assert O.pack_append_buffer(cache, "k", 8).size == 3 * 2 * 64 * 256


def test_folding_appended_tokens_gives_the_cache_of_the_longer_context():
    """Sec. III-A: context + appended rows, folded, is exactly what reorder_quantize builds from the longer
    context whose completed chunks are FP16 chunks: plans, every class array, the byte images and the attention.
    Catches: rows folded in front of the remainder, a completed chunk given another bitwidth, rows of one
    sequence folded into another, rows left in the append list."""
    chunk = 16
    w = workloads.small("fold", 3, 4, 2, [70, 33, 125], chunk, 32, mix=(0.25, 0.35, 0.4), seed_offset=31)
    ks, vs = _seqs(w)
    bits = workloads.chunk_bits(w)
    grow = [21, 0, 40]                                    # 70 + 21 = 91 completes chunk 4; 125 + 40 completes 3 chunks
    cache = O.reorder_quantize(ks, vs, bits, chunk, 32)
    new_k = [np.zeros((2, 0, 128), np.float16) for _ in range(3)]
    new_v = [np.zeros((2, 0, 128), np.float16) for _ in range(3)]
    for step in range(max(grow)):
        kn, vn = _new_tokens(w, 300 + step)
        active = [step < grow[b] for b in range(3)]
        O.append_tokens(cache, kn, vn, active)
        for b in range(3):
            if active[b]:
                new_k[b] = np.concatenate([new_k[b], kn[b][:, None, :]], axis=1)
                new_v[b] = np.concatenate([new_v[b], vn[b][:, None, :]], axis=1)
    q = workloads.query(w, 0)
    before, lse_before = O.decode_attention(q, cache)
    O.fold_appended(cache)
    long_k = [np.concatenate([ks[b], new_k[b]], axis=1) for b in range(3)]
    long_v = [np.concatenate([vs[b], new_v[b]], axis=1) for b in range(3)]
    long_bits = [np.concatenate([bits[b], np.full((w.seq_lens[b] + grow[b]) // chunk - len(bits[b]), 16, np.uint8)])
                 for b in range(3)]
    assert [len(x) for x in long_bits] == [5, 2, 10]
    fresh = O.reorder_quantize(long_k, long_v, long_bits, chunk, 32)
    assert cache.seq_lens == fresh.seq_lens == [91, 33, 165]
    for b in range(3):
        assert cache.app_k[b].shape[1] == 0 and cache.app_v[b].shape[1] == 0
        assert np.array_equal(cache.bits[b], fresh.bits[b])
        assert np.array_equal(cache.plans[b].perm, fresh.plans[b].perm)
        assert cache.plans[b].class_chunks == fresh.plans[b].class_chunks
        assert cache.plans[b].class_tokens == fresh.plans[b].class_tokens and cache.plans[b].tail == fresh.plans[b].tail
        for c in range(O.NUM_CLASSES):
            a, f = cache.seqs[b][c], fresh.seqs[b][c]
            assert a.n_tokens == f.n_tokens
            for name in ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "k_raw", "v_raw"):
                x, y = getattr(a, name), getattr(f, name)
                assert (x is None) == (y is None)
                if x is not None:
                    assert np.array_equal(np.ascontiguousarray(x).view(np.uint8), np.ascontiguousarray(y).view(np.uint8)), name
    for c in range(O.NUM_CLASSES):
        for which in ("k", "v"):
            for quads in (False, True):
                assert np.array_equal(O.pack_class_buffer(cache, c, which, quads), O.pack_class_buffer(fresh, c, which, quads))
    after, lse_after = O.decode_attention(q, cache)
    fr, lse_fr = O.decode_attention(q, fresh)
    np.testing.assert_array_equal(after, fr)
    np.testing.assert_allclose(after, before, rtol=0, atol=1e-13)      # folding does not change the attention
    np.testing.assert_allclose(lse_after, lse_before, rtol=0, atol=1e-13)
    # the appended rows sit behind the old remainder: the last rows of the FP16 list are the new tokens
    for b in (0, 2):
        assert np.array_equal(cache.seqs[b][O.FP16_CLASS].k_raw[:, -grow[b]:], new_k[b])


def test_fp16_runs_with_room_to_grow_are_the_runs_followed_by_zero_blocks():
    """pack_class_buffer(reserve=...): the layout a cache has when appended rows are to be folded into it later.
    Catches: room counted in blocks instead of tokens, room given to another class, a run without tokens that gets
    no room, spare blocks in front of the run."""
    w = workloads.small("reserve", 3, 2, 2, [64 + 10, 8, 200], 8, 32, mix=(0.3, 0.3, 0.4), seed_offset=37)
    ks, vs = _seqs(w)
    bits = [x.copy() for x in workloads.chunk_bits(w)]
    bits[1][:] = 2                                        # sequence 1: no FP16 tokens at all (8 tokens = one INT2 chunk)
    bits[0][:] = 2
    bits[0][0] = 16                                       # sequence 0: one FP16 chunk + the 2-token remainder
    cache = O.reorder_quantize(ks, vs, bits, 8, 32)
    assert cache.seqs[1][O.FP16_CLASS].n_tokens == 0 and cache.seqs[0][O.FP16_CLASS].n_tokens == 10
    bb = 64 * 256
    # 10 tokens + room for 50 still fit the run's one block; + 60 need a second one
    for reserve, spare0 in (([50, 70, 0], 0), ([60, 1, 5], 1)):
        for which, quads in (("k", False), ("v", False), ("v", True)):
            plain = O.pack_class_buffer(cache, O.FP16_CLASS, which, quads)
            roomy = O.pack_class_buffer(cache, O.FP16_CLASS, which, quads, reserve=reserve)
            pos_p = pos_r = 0
            for b in range(3):
                n = cache.seqs[b][O.FP16_CLASS].n_tokens
                used = -(-n // 64)
                total = -(-(n + reserve[b]) // 64)
                if b == 0:
                    assert total - used == spare0
                for h in range(2):
                    assert np.array_equal(roomy[pos_r:pos_r + used * bb], plain[pos_p:pos_p + used * bb])
                    assert not roomy[pos_r + used * bb:pos_r + total * bb].any()
                    pos_p += used * bb
                    pos_r += total * bb
            assert pos_p == plain.size and pos_r == roomy.size
            # other classes take no room
            assert np.array_equal(O.pack_class_buffer(cache, 0, which, quads, reserve=reserve),
                                  O.pack_class_buffer(cache, 0, which, quads))
    # sequence 1 has no FP16 tokens: room for 70 is two blocks per head, room for 1 is one
    assert O.pack_class_buffer(cache, O.FP16_CLASS, "k", reserve=[0, 70, 0]).size - O.pack_class_buffer(cache, O.FP16_CLASS, "k").size == 2 * 2 * bb


def test_page_gather_by_hand_and_round_trip():
    """gather_pages against a table typed out by hand, and as the inverse of a scatter into shuffled pages."""
    # 3 pages of 2 tokens, 1 head, D = 1: page p, slot s holds the value 10 p + s
    pages = np.array([[[[0.0], [1.0]]], [[[10.0], [11.0]]], [[[20.0], [21.0]]]], dtype=np.float16)
    got = O.gather_pages(pages, [2, 0, 1], 5)                       # tokens 0,1 from page 2; 2,3 from page 0; 4 from page 1
    assert got[0, :, 0].tolist() == [20.0, 21.0, 0.0, 1.0, 10.0]
    rng = np.random.default_rng(5)
    hkv, t, d, ps = 2, 37, 8, 4
    k = rng.standard_normal((hkv, t, d)).astype(np.float16)
    npages = (t + ps - 1) // ps
    table = rng.permutation(npages + 3)[:npages]                    # pages anywhere in a larger pool
    pool = np.zeros((npages + 3, hkv, ps, d), dtype=np.float16)
    for tok in range(t):
        pool[table[tok // ps], :, tok % ps, :] = k[:, tok, :]
    assert np.array_equal(O.gather_pages(pool, table, t), k)
