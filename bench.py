"""Benchmark of the chunk-level KV cache computation hot path on one MI355X.

One "step" is one pass of the whole path for one attention layer of the headline
workload (Llama2-13B-shaped, 128K context, 512-token chunks, G=64): the prefill
side once (reorder + quantize + pack of the layer's fp16 K/V), then the decode
side once per generated token (single-query attention over the packed cache);
the paper generates 128 output tokens per request (Sec. IV, Experiment Setup),
so a step holds 128 decode calls.  Several cache copies (at least 768 MB in total)
take turns, so no call reads data that an earlier call left in the last-level cache.  Inputs are resident in
HBM before the timed region.  `value` is the mean decode-attention time per layer
call: HIP events recorded on the launch stream around the decode calls of every
timed step, divided by the number of calls; the reorder+quantize time is reported
next to it.

After the timed steps of the headline workload, a short pass over each of the other four benchmark
configurations fills the `configs` array (same protocol, fewer steps; configuration 2 takes its cache copies
from six distinct layers, as the 32 layers of a model would), each with the parity error of sampled heads
against the CPU oracle.

Prints ONE JSON line: metric, value (us per decode call), roofline (achieved GB/s of that call against the
8 TB/s HBM peak, HBM traffic from the committed counter runs), cpu_baseline (the numpy oracle on a sample of
the same workload) and configs (all five configurations).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "decode-attention us/layer and achieved HBM GB/s (% of peak) at 128K ctx"
MIN_ROTATION_BYTES = 768 << 20     # cache copies that take turns hold at least this much: three times the last-level cache


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([int(p.get("num_threads", 1)) for p in threadpool_info()] or [1])
    except Exception:
        return 1


def oracle_sample(w, layer_of, bits, q_of, gpu_out_of, heads):
    """Runs the numpy oracle on the (cache copy, sequence, kv head) units in `heads`, times it, and compares
    the GPU output on them.  Returns (reorder+quantize seconds, attention seconds, worst relative error)."""
    from oracle import cocktail_oracle as O
    import workloads
    t_rq = t_att = 0.0
    worst = 0.0
    rep = w.num_q_heads // w.num_kv_heads
    for copy, b, h in heads:
        kh, vh = workloads.kv_head(w, layer_of(copy), b, h)
        t0 = time.perf_counter()
        oc = O.reorder_quantize([kh[None]], [vh[None]], [bits[b]], w.chunk_size, w.group_size)
        t1 = time.perf_counter()
        ref, _ = O.decode_attention(q_of(copy)[b:b + 1, h * rep:(h + 1) * rep], oc)
        t2 = time.perf_counter()
        t_rq += t1 - t0
        t_att += t2 - t1
        for r in range(rep):
            got = gpu_out_of(copy)[b, h * rep + r].astype(np.float64)
            worst = max(worst, float(np.abs(got - ref[0, r]).max() / np.abs(ref[0, r]).max()))
    return t_rq, t_att, worst


def measured_traffic(workload_name):
    """HBM bytes per decode call and the file they come from: the committed rocprofv3 counter summary of this
    workload under profiles/ ((None, None) if there is none).  Not measured in this run."""
    for kernel in ("decode_attention", "decode_quads"):
        name = f"{kernel}_{workload_name}_hbm_traffic.txt"
        try:
            with open(os.path.join(ROOT, "profiles", name)) as f:
                for line in f:
                    if line.startswith("traffic_bytes_per_call:"):
                        return float(line.split(":", 1)[1].split()[0]), "profiles/" + name
        except OSError:
            pass
    return None, None


def run_config(cfg, steps, warmup, ntok, workers_arg, decode_only, cpu_heads, calibrate_copy=False, vector_alu_only=False):
    """Times one benchmark configuration; returns (entry for the `configs` array, details for the headline)."""
    import torch
    import paper_2503_23294_amd as ck
    import workloads

    dev = torch.device("cuda:0")
    w = workloads.config(cfg)
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    bits = workloads.chunk_bits(w)
    workers = workers_arg or ck.cocktail_default_workers(shape, vector_alu_only)
    plan = ck.cocktail_plan(shape, w.seq_lens, np.concatenate(bits), workers, vector_alu_only=vector_alu_only)
    packed = int(plan.sizes.packed_bytes)
    # enough cache copies that a call never finds its data in the 256 MB last-level cache
    ncopies = min(max(2, -(-MIN_ROTATION_BYTES // max(packed, 1))), 64)
    # a model's layers hold different data: copies come from distinct layers where the configuration has them
    nlayers = min(ncopies, w.num_layers)
    layer_of = (lambda i: (i * max(w.num_layers // nlayers, 1)) % w.num_layers) if nlayers > 1 else (lambda i: 0)
    t0 = time.perf_counter()
    src, qs, q_host = {}, {}, {}
    for i in range(ncopies):
        layer = layer_of(i)
        if layer not in src:
            k, v = workloads.kv_flat(w, layer, threads=16)
            src[layer] = (torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev))
            src_bytes = int(k.nbytes + v.nbytes)
            del k, v
            q_host[layer] = workloads.query(w, layer)
            qs[layer] = torch.from_numpy(q_host[layer]).to(dev)
    log(f"{w.name}: generated {len(src)} layer(s) of fp16 K/V, {src_bytes / 1e9:.2f} GB each, in "
        f"{time.perf_counter() - t0:.1f} s; {ncopies} cache copies")
    caches = [ck.PackedCache(plan, dev) for _ in range(ncopies)]
    outs = [torch.empty_like(qs[layer_of(i)]) for i in range(ncopies)]
    lse = torch.empty((w.batch, w.num_q_heads), dtype=torch.float32, device=dev)

    qo_bytes = 2 * w.batch * w.num_q_heads * w.head_dim * 2
    decode_bytes = packed + qo_bytes                        # algorithmic bytes of one decode call
    rq_bytes = src_bytes + packed                           # read fp16 K,V once, write the packed cache

    def rq(i):
        k_dev, v_dev = src[layer_of(i % ncopies)]
        ck.cocktail_reorder_quantize(caches[i % ncopies], k_dev, v_dev, ragged=True)

    def dec(i):
        ck.cocktail_decode_attention(caches[i % ncopies], qs[layer_of(i % ncopies)], 0.0, outs[i % ncopies], lse)

    for i in range(ncopies):
        rq(i)
    torch.cuda.synchronize()

    def step(i, ev=None):
        if ev is not None:
            ev[0].record()
        if not decode_only:
            rq(i)
        if ev is not None:
            ev[1].record()
        for j in range(ntok):
            dec(i + 1 + j)
        if ev is not None:
            ev[2].record()

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    if calibrate_copy:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, ev[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    rq_us = np.array([e[0].elapsed_time(e[1]) for e in ev]) * 1e3
    # one event pair around the decode calls of a step: mean time per call in a running decode loop
    dec_us = np.array([e[1].elapsed_time(e[2]) for e in ev]) * 1e3 / ntok
    dec_mean = float(dec_us.mean())
    gbps = decode_bytes / (dec_mean * 1e-6) / 1e9
    # The dominant kernel alone, live: an event recorded by the library between the partial-state kernel and the
    # merge (cocktail_decode_attention_marked), one event triple per call, outside the timed region above (the
    # extra record sits between the two kernels and delays the merge, so only start -> between is used: the
    # partial-state kernel with its launch; the merge kernel's time is in the rocprofv3 summaries under profiles/).
    nmark = min(ntok, 64)
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(nmark)]
    for trip in marks:
        trip[1].record()                                    # torch creates the handle at the first record
    torch.cuda.synchronize()
    for i in range(8):
        dec(i)
    for j, trip in enumerate(marks):
        i = j % ncopies
        trip[0].record()
        ck.cocktail_decode_attention_marked(caches[i], qs[layer_of(i)], trip[1], outs[i], lse)
        trip[2].record()
    torch.cuda.synchronize()
    kernel_us = float(np.mean([t[0].elapsed_time(t[1]) for t in marks]) * 1e3)
    for c in caches:
        ck.cocktail_decode_check(c)                         # every call attended to every token exactly once
    gpu_out = [o.cpu().numpy() for o in outs]

    entry = {
        "workload": w.name, "decode_us": dec_mean, "decode_us_median_step": float(np.median(dec_us)),
        "decode_us_min_step": float(dec_us.min()), "decode_algorithmic_bytes": decode_bytes,
        "gbps": gbps, "frac_of_hbm_peak": gbps / HBM_PEAK_GBPS,
        "partial_state_kernel_us": kernel_us,
        "partial_state_kernel_frac_of_hbm_peak": decode_bytes / (kernel_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        "reorder_quantize_us": None if decode_only else float(rq_us.mean()),
        "reorder_quantize_bytes": rq_bytes,
        "reorder_quantize_gbps": None if decode_only else rq_bytes / (float(rq_us.mean()) * 1e-6) / 1e9,
        "kernel": "decode_quads_kernel" if int(plan.sizes.v_layout) == 1 else "decode_attention_kernel",
        "kernel_family": ("four query heads per wave on 4x4x4 matrix instructions"
                          + (", two waves per workgroup sharing their K/V units through shared memory"
                             if w.num_q_heads // w.num_kv_heads > 4 else "")) if int(plan.sizes.v_layout) == 1
                         else "one query head per wave on the vector ALU (no matrix instructions)",
        "cache_copies": ncopies, "distinct_layers": len(src), "steps": steps, "decode_calls_per_step": ntok,
    }
    base = None
    if cpu_heads > 0:
        rng = np.random.default_rng(cfg)
        units = [(c, b, h) for c in range(min(ncopies, max(len(src), 1))) for b in range(w.batch)
                 for h in range(w.num_kv_heads) if w.seq_lens[b] > 0]
        pick = sorted(units[i] for i in rng.choice(len(units), size=min(cpu_heads, len(units)), replace=False))
        t_rq, t_att, worst = oracle_sample(w, layer_of, bits, lambda c: q_host[layer_of(c)], lambda c: gpu_out[c], pick)
        entry["parity_max_rel_err"] = worst
        entry["parity_sample"] = f"{len(pick)} (layer, sequence, kv head) units against the CPU oracle"
        assert worst <= 2e-3, f"{w.name}: GPU output disagrees with the oracle on the sampled heads: {worst:.3e}"
        total_units = sum(1 for b in range(w.batch) for _ in range(w.num_kv_heads))
        scale = total_units / len(pick)
        base = {
            "value": t_att * scale * 1e6, "unit": "us/layer", "cores": blas_threads(), "kind": "oracle",
            "host_cpus": os.cpu_count(),
            "sample": f"{len(pick)} of {total_units} (sequence, kv head) units of the same workload, scaled "
                      f"linearly; cores = BLAS threads of the matrix products, the quantizer and the gathers are "
                      f"single-threaded numpy; reorder+quantize on the same sample: {t_rq * scale * 1e6:.0f} us/layer",
            "reorder_quantize_us": t_rq * scale * 1e6,
        }
    detail = {"w": w, "plan": plan, "workers": workers, "wall": wall, "decode_bytes": decode_bytes, "cpu_baseline": base,
              "class_tokens": [int(x) for x in plan.class_tokens.sum(axis=0)]}
    del caches, src, qs, outs
    torch.cuda.empty_cache()
    return entry, detail


def paged_reorder_quantize(cfg, page_sizes, reps=8):
    """Times reorder+quantize reading K and V from a paged cache (pages shuffled over the pool) for one
    configuration; checks that the packed cache equals the one made from the flat source, byte for byte."""
    import torch
    import paper_2503_23294_amd as ck
    import workloads

    dev = torch.device("cuda:0")
    w = workloads.config(cfg)
    shape = ck.make_shape(w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.chunk_size, w.group_size)
    plan = ck.cocktail_plan(shape, w.seq_lens, np.concatenate(workloads.chunk_bits(w)), ck.cocktail_default_workers(shape))
    k, v = workloads.kv_flat(w, 0, threads=16)
    src_bytes = int(k.nbytes + v.nbytes)
    k_dev, v_dev = torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev)
    del k, v
    ref, cache = ck.PackedCache(plan, dev), ck.PackedCache(plan, dev)
    ck.cocktail_reorder_quantize(ref, k_dev, v_dev, ragged=True)
    off = workloads.seq_token_offsets(w)
    h, d = w.num_kv_heads, w.head_dim
    out = []
    for ps in page_sizes:
        need = [-(-t // ps) for t in w.seq_lens]
        total = sum(need)
        g = torch.Generator(device="cpu").manual_seed(ps)
        ids = torch.randperm(total, generator=g).to(dev)
        table = torch.full((w.batch, max(need)), -1, dtype=torch.int32, device=dev)
        pools = []
        for flat in (k_dev, v_dev):
            pool = torch.zeros((total, h, ps, d), dtype=torch.float16, device=dev)
            pos = 0
            for b, t in enumerate(w.seq_lens):
                if t == 0:
                    continue
                seq = flat[int(off[b]) * h * d:int(off[b + 1]) * h * d].view(h, t, d)
                padded = torch.zeros((h, need[b] * ps, d), dtype=torch.float16, device=dev)
                padded[:, :t] = seq
                pool[ids[pos:pos + need[b]]] = padded.view(h, need[b], ps, d).permute(1, 0, 2, 3)
                table[b, :need[b]] = ids[pos:pos + need[b]].to(torch.int32)
                pos += need[b]
                del padded
            pools.append(pool)
        for c in cache.k + cache.v:
            c.zero_()
        ck.cocktail_reorder_quantize_paged(cache, pools[0], pools[1], table)
        torch.cuda.synchronize()
        for a, b_ in zip(cache.k + cache.v, ref.k + ref.v):
            assert torch.equal(a, b_), "paged source: packed cache differs from the one made from the flat source"
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        for i in range(reps):
            ev[i].record()
            ck.cocktail_reorder_quantize_paged(cache, pools[0], pools[1], table)
        ev[reps].record()
        torch.cuda.synchronize()
        us = ev[0].elapsed_time(ev[reps]) * 1e3 / reps
        nbytes = src_bytes + int(plan.sizes.packed_bytes)
        out.append({"page_size": ps, "us": us, "gbps": nbytes / (us * 1e-6) / 1e9,
                    "frac_of_hbm_peak": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS})
        del pools, table
    del k_dev, v_dev, ref, cache
    torch.cuda.empty_cache()
    return out


def stream_read_ceiling(nbytes):
    """The rate of a plain 128-bit streaming read of about `nbytes` over two alternating buffers (GB/s)."""
    import torch
    import paper_2503_23294_amd as ck
    dev = torch.device("cuda:0")
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_bytes = max(nbytes, 1 << 28)
    bufs = [torch.zeros(probe_bytes, dtype=torch.uint8, device=dev) for _ in range(2)]
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(33)]
    for i in range(4):
        read = ck.cocktail_stream_read_probe(bufs[i % 2], sink)
    torch.cuda.synchronize()
    for i in range(32):
        pe[i].record()
        ck.cocktail_stream_read_probe(bufs[i % 2], sink)
    pe[32].record()
    torch.cuda.synchronize()
    stream_us = pe[0].elapsed_time(pe[32]) * 1e3 / 32
    return read / (stream_us * 1e-6) / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload: benchmark configuration 1..5 (headline: 4); 6..9 = extra shapes (8 query heads per kv head; head_dim 64; INT8 mixes)")
    ap.add_argument("--workers", type=int, default=0, help="decode workgroups (0 = library default)")
    ap.add_argument("--cpu-heads", type=int, default=32, help="kv heads the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--decode-only", action="store_true", help="steps run decode attention only (for profiling)")
    ap.add_argument("--tokens-per-step", type=int, default=128, help="decode calls per step (output tokens per request)")
    ap.add_argument("--other-configs", type=int, default=1,
                    help="1 = also run a short pass over the other four configurations (the `configs` array)")
    ap.add_argument("--vector-alu-only", action="store_true",
                    help="plan grouped-query shapes for the kernel without matrix instructions (one query head per wave)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy, the known-size kernel that scales the HBM traffic counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives or sharding are part of it); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    ntok = max(1, args.tokens_per_step)
    head, d = run_config(args.config, args.steps, args.warmup, ntok, args.workers, args.decode_only, args.cpu_heads,
                         args.calibrate_copy, args.vector_alu_only)
    w, plan = d["w"], d["plan"]
    stream_gbps = stream_read_ceiling(d["decode_bytes"])
    traffic, traffic_source = measured_traffic(w.name)
    gbps = head["gbps"]
    configs = [head]
    if args.other_configs:
        for cfg in (1, 2, 3, 5, 4):
            if cfg == args.config:
                continue
            entry, _ = run_config(cfg, steps=6, warmup=2, ntok=64, workers_arg=args.workers, decode_only=False, cpu_heads=2)
            entry["frac_of_stream_read"] = entry["gbps"] / stream_gbps
            if entry["kernel"] == "decode_quads_kernel":
                # the same shape on the kernel without matrix instructions (one query head per wave), for reference
                alt, _ = run_config(cfg, steps=3, warmup=1, ntok=32, workers_arg=args.workers, decode_only=True, cpu_heads=1,
                                    vector_alu_only=True)
                entry["vector_alu_only"] = {"decode_us": alt["decode_us"], "frac_of_hbm_peak": alt["frac_of_hbm_peak"],
                                            "parity_max_rel_err": alt["parity_max_rel_err"]}
            configs.append(entry)
        configs.sort(key=lambda e: e["workload"])
    head["frac_of_stream_read"] = gbps / stream_gbps
    paged = paged_reorder_quantize(args.config, (16, 256)) if args.other_configs and not args.decode_only else None

    result = {
        "metric": METRIC, "value": head["decode_us"], "unit": "us/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": d["wall"] / args.steps * 1e3, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "q_heads": w.num_q_heads, "kv_heads": w.num_kv_heads,
                   "head_dim": w.head_dim, "context": list(w.seq_lens), "chunk_size": w.chunk_size,
                   "group_size": w.group_size,
                   "class_tokens_int2_int4_int8_fp16": d["class_tokens"],
                   "decode_workgroups": d["workers"], "decode_calls_per_step": ntok, "cache_copies": head["cache_copies"],
                   "kernel_family": "one query head per wave on the vector ALU (no matrix instructions)"
                   if head["kernel"] == "decode_attention_kernel" else
                   "four query heads per wave on 4x4x4 matrix instructions (grouped-query shapes)",
                   "step": "reorder+quantize once, then one decode-attention call per output token"
                   if not args.decode_only else "decode attention only"},
        "decode_us_median_step": head["decode_us_median_step"], "decode_us_min_step": head["decode_us_min_step"],
        "achieved_gbps": gbps, "pct_of_hbm_peak": 100.0 * gbps / HBM_PEAK_GBPS,
        "decode_algorithmic_bytes": d["decode_bytes"],
        "stream_read_gbps": stream_gbps, "frac_of_stream_read": gbps / stream_gbps,
        "reorder_quantize_us": head["reorder_quantize_us"], "reorder_quantize_gbps": head["reorder_quantize_gbps"],
        "reorder_quantize_bytes": head["reorder_quantize_bytes"],
        "reorder_quantize_from_pages": paged,
        # the dominant kernel: the partial-state kernel, which streams the packed cache; its average duration
        # from HIP events on the launch stream (one recorded by the library between the call's two kernels)
        "roofline": {"bound": "hbm", "achieved": d["decode_bytes"] / (head["partial_state_kernel_us"] * 1e-6) / 1e9,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": head["partial_state_kernel_frac_of_hbm_peak"],
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": head["kernel"], "kernel_avg_us": head["partial_state_kernel_us"],
                     "whole_call": {"us": head["decode_us"], "achieved": gbps, "frac": gbps / HBM_PEAK_GBPS,
                                    "kernels": head["kernel"] + " + decode_merge_kernel"}},
        "configs": configs,
    }
    if d["cpu_baseline"] is not None:
        result["cpu_baseline"] = d["cpu_baseline"]
        result["parity_max_rel_err_on_cpu_sample"] = head["parity_max_rel_err"]
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
