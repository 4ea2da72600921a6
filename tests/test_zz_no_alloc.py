"""The entry point that allocates nothing (cocktail_decode_attention_static) against cocktail_decode_attention.

Collected last on purpose (the file name sorts behind the other test files): it is the only test that uses the
workspace built into the library, and a failure here must not hide the parity tests.
"""
import numpy as np
import pytest
import torch

import workloads
import paper_2503_23294_amd as ck
from paper_2503_23294_amd import _lib

TOL = 2e-3      # max_d |a - b| / max_d |b| per (sequence, query head): the bar of the parity tests


def _prepare(w, workers, dev):
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = np.concatenate(workloads.chunk_bits(w))
    plan = ck.cocktail_plan(shape, w.seq_lens, bits, workers)
    cache = ck.PackedCache(plan, dev)
    k, v = workloads.kv_flat(w, 0)
    ck.cocktail_reorder_quantize(cache, torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev), ragged=True)
    q = torch.from_numpy(workloads.query(w, 0)).to(dev)
    return cache, q


@pytest.mark.gpu
@pytest.mark.parametrize("rep", [1, 4])
def test_static_workspace_entry_point_matches_the_regular_one(rep):
    assert torch.cuda.is_available(), "this test needs the MI355X"
    dev = torch.device("cuda:0")
    # two calls in a row on the library's one workspace, the second with a smaller input: whatever the first
    # call left there must not leak into the second
    big = workloads.small(f"static_big_r{rep}", 3, 2 * rep, 2, [5000, 2100, 3300], 64, 32, mix=(0.2, 0.4, 0.4),
                          seed_offset=800 + rep)
    small = workloads.small(f"static_small_r{rep}", 1, 2 * rep, 2, [64 * 3 + 11], 32, 32, mix=(0.3, 0.3, 0.4),
                            seed_offset=810 + rep)
    for w, workers in ((big, 48), (small, 5)):
        print(f"[no-alloc] {w.name}", flush=True)
        cache, q = _prepare(w, workers, dev)
        assert int(cache.plan.sizes.workspace_bytes) <= _lib.STATIC_WORKSPACE_BYTES
        ref, ref_lse = ck.cocktail_decode_attention(cache, q)
        ck.cocktail_decode_check(cache)
        out = torch.full_like(ref, float("nan"))
        lse = torch.full_like(ref_lse, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        ck.cocktail_decode_attention_static(cache, q, 0.0, out, lse)
        assert torch.cuda.memory_allocated() == before
        ck.cocktail_decode_check(cache, static_workspace=True)      # also waits for the stream
        a, b = out.float(), ref.float()
        err = ((a - b).abs().amax(dim=2) / b.abs().amax(dim=2)).max().item()
        assert np.isfinite(err) and err <= TOL, f"{w.name}: max relative deviation {err:.3e}"
        assert torch.allclose(lse, ref_lse, rtol=0, atol=1e-4 * max(1.0, float(ref_lse.abs().max())))
        # the regular entry point still works after it, on its own workspace
        again, _ = ck.cocktail_decode_attention(cache, q)
        torch.cuda.synchronize()
        err = ((again.float() - b).abs().amax(dim=2) / b.abs().amax(dim=2)).max().item()
        assert err <= TOL


def test_static_workspace_entry_point_rejects_plans_beyond_its_size():
    """Host-side check, before any HIP call: runs without a GPU."""
    import ctypes as C
    sh = ck.make_shape(1, 1, 1, 128, 4096, 32)
    plan = ck.cocktail_plan(sh, [4096 * 640], np.full(640, 4, np.uint8), 1 << 15)   # 40960 blocks: a partial per worker
    assert int(plan.sizes.workspace_bytes) > _lib.STATIC_WORKSPACE_BYTES
    cache = _lib.Cache()
    cache.plan_host = plan.blob.ctypes.data
    cache.plan_dev = 4096
    L = _lib.lib()
    assert L.cocktail_decode_attention_static(C.byref(sh), 16, C.byref(cache), 0.0, 16, None, None) == _lib.ENOSPACE
    assert b"built-in" in L.cocktail_last_error()
    assert L.cocktail_decode_attention_static(C.byref(sh), None, C.byref(cache), 0.0, 16, None, None) == _lib.EINVAL
