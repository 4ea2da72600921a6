"""Tuning aid: when does every decode workgroup start and end inside one cocktail_decode_attention call?

Needs a build of the library with per-worker time stamps, made on the build machine with
    python -m paper_2503_23294_amd.build --out paper_2503_23294_amd/libcocktail_trace.so -DCOCKTAIL_TRACE
and is then run on the GPU as
    COCKTAIL_LIB=paper_2503_23294_amd/libcocktail_trace.so python -m paper_2503_23294_amd.worker_trace --config 2
(the package loads the library named by COCKTAIL_LIB when it is imported, which `python -m` does before this
module runs, so the variable has to be set by the caller)
It prints the start and end times of the workers (microseconds from the first start), per bitwidth class and
per group of workers that share a pool, next to the time a plain stream read of the packed bytes would take:
the split of a call into start-up, streaming and the tail between the first and the last worker to finish.
"""
from __future__ import annotations

import argparse
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
TRACE_LIB = os.path.join(HERE, "libcocktail_trace.so")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 1..5")
    ap.add_argument("--workers", type=int, default=0)
    args = ap.parse_args()
    if not os.path.exists(TRACE_LIB):
        sys.exit(f"{TRACE_LIB} is missing; build it first (see the module docstring)")
    sys.path.insert(0, os.path.dirname(HERE))
    from paper_2503_23294_amd import _lib
    if os.path.abspath(_lib.LIB_PATH) != TRACE_LIB:
        sys.exit(f"the package loaded {_lib.LIB_PATH}; run with COCKTAIL_LIB={TRACE_LIB} (see the module docstring)")
    import numpy as np
    import torch
    import paper_2503_23294_amd as ck
    import workloads

    dev = torch.device("cuda:0")
    w = workloads.config(args.config)
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    workers = args.workers or ck.cocktail_default_workers(shape)
    plan = ck.cocktail_plan(shape, w.seq_lens, np.concatenate(workloads.chunk_bits(w)), workers)
    workers = int(plan.sizes.num_workers)   # a short context gets fewer workers than asked for
    tokens, hkv = sum(w.seq_lens), w.num_kv_heads
    # timing only: Gaussian noise of the right shape stands in for the workload's K, V and q
    k = torch.randn(hkv * tokens * w.head_dim, device=dev, dtype=torch.float16)
    v = torch.randn(hkv * tokens * w.head_dim, device=dev, dtype=torch.float16)
    q = torch.randn(w.batch, w.num_q_heads, w.head_dim, device=dev, dtype=torch.float16)
    ncop = min(max(2, -(-(768 << 20) // int(plan.sizes.packed_bytes))), 8)
    caches = [ck.PackedCache(plan, dev) for _ in range(ncop)]
    wsb = (int(plan.sizes.workspace_bytes) + 255) // 256 * 256
    for c in caches:
        c.workspace = torch.zeros(wsb + workers * 32, dtype=torch.uint8, device=dev)   # the tracing build writes 32 B per worker behind the workspace
        ck.cocktail_reorder_quantize(c, k, v, ragged=True)
    torch.cuda.synchronize()
    for i in range(4 * ncop):
        ck.cocktail_decode_attention(caches[i % ncop], q)
    torch.cuda.synchronize()
    tr = caches[ncop - 1].workspace[wsb:].cpu().numpy().view(np.uint64).reshape(workers, 4).astype(np.int64)
    t0 = tr[:, 0].min()
    st, en = (tr[:, 0] - t0) / 100.0, (tr[:, 1] - t0) / 100.0      # the stamps count 100 MHz ticks
    f = lambda name, i=0: ck.cocktail_plan_field(plan, name, i)
    rec_words = f("sizeof_worker_rec") // 4
    recs = np.frombuffer(plan.blob.tobytes(), dtype=np.int32, count=rec_words * workers,
                         offset=f("off_worker_rec")).reshape(workers, rec_words)
    own_blocks, cls, group = recs[:, 1] - recs[:, 0], recs[:, 6], recs[:, 12]
    packed = int(plan.sizes.packed_bytes)
    print(f"{w.name}: {workers} workers, {packed / 1e6:.1f} MB packed; a stream read at 6.5 TB/s takes {packed / 6.5e6:.1f} us")
    print(f"  start  min/median/max {st.min():.2f} / {np.median(st):.2f} / {st.max():.2f} us")
    print(f"  end    min/p10/median/p90/max {en.min():.1f} / {np.percentile(en, 10):.1f} / {np.median(en):.1f} / "
          f"{np.percentile(en, 90):.1f} / {en.max():.1f} us   (workers without an own range: {int((own_blocks == 0).sum())})")
    for c, name in enumerate(("INT2", "INT4", "INT8", "FP16")):
        m = (cls == c) & (own_blocks > 0)
        if m.any():
            print(f"  {name}: {int(m.sum())} workers, {np.median(own_blocks[m]):.0f} own blocks each, end min/median/max "
                  f"{en[m].min():.1f} / {np.median(en[m]):.1f} / {en[m].max():.1f} us")
    # duration by own class and by the class of the SIMD mate (workgroup i shares a SIMD with workgroup i + P/2)
    if workers % 2 == 0:
        mate = np.roll(cls, -workers // 2)
        names = ("INT2", "INT4", "INT8", "FP16")
        print("  own ranges: worker end (median us) by own class (rows) and SIMD mate's class (columns), workers counted")
        for c in range(4):
            cells = []
            for m in range(4):
                sel = (cls == c) & (mate == m) & (own_blocks > 0)
                cells.append(f"{names[m]} {np.median(en[sel]):6.1f} ({int(sel.sum()):4d})" if sel.any() else f"{names[m]}      - (   0)")
            if ((cls == c) & (own_blocks > 0)).any():
                print(f"    {names[c]}: " + "   ".join(cells))
    ng = int(group.max()) + 1
    gend = np.array([en[group == g].max() for g in range(ng)])
    gfirst = np.array([en[group == g].min() for g in range(ng)])
    print(f"  {ng} groups: last member ends min/median/p90/max {gend.min():.1f} / {np.median(gend):.1f} / "
          f"{np.percentile(gend, 90):.1f} / {gend.max():.1f} us; spread inside a group median/max "
          f"{np.median(gend - gfirst):.2f} / {(gend - gfirst).max():.2f} us")


if __name__ == "__main__":
    main()
