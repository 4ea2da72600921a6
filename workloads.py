"""Seeded synthetic inputs for the chunk-level KV cache computation path.

This module only draws random tensors and chunk bitwidth labels.  It holds none
of the method's arithmetic (no quantisation, packing, reordering or attention),
so both the CPU oracle's tests and the HIP path's tests/bench may import it.

The workloads stand in for the long-context evaluation the paper runs (Sec. IV,
"Experiment Setup": Llama2-7B/13B, Mistral-7B, Longchat-7B on a long-context
benchmark): shapes follow those models' attention geometry, and the share of
chunks kept at each bitwidth follows the paper's observation that only a few
chunks are relevant to the query (Sec. I, Fig. 1).  Nothing of that benchmark's
items is reproduced here: every tensor is Gaussian noise.

Recipe (per config `c`, layer `l`, sequence `b`, head `h`):
  K[b,h] ~ N(0,1) [T_b, D] fp16; 4 channels per (layer, kv-head), drawn without
           replacement, are multiplied by 10 for every token (key outliers);
  V[b,h] ~ N(0,1) [T_b, D] fp16;   q[b,hq] ~ N(0,1) [D] fp16;
  chunk bits: iid per chunk with the config's P(FP16, INT4, INT2) (test shapes may add an INT8
           share: P(FP16, INT8, INT4, INT2)), shared by
           all layers and heads of a sequence (the bitwidth configuration comes
           from text chunks, Sec. III-B);  config 5 draws a Dirichlet(1,1,1)
           mix per sequence and forces sequence 0 to all-FP16, 1 to all-INT2.
Every draw is keyed by (BASE_SEED, config, layer, b, h, tag) so any single head
can be regenerated without producing the whole tensor.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 250323294

_TAG_K, _TAG_V, _TAG_Q, _TAG_BITS, _TAG_OUTLIER, _TAG_LEN, _TAG_MIX, _TAG_EMB = range(8)


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic workload (one attention layer call)."""
    name: str
    config: int                 # 1..5, index into the benchmark's config list
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    chunk_size: int
    group_size: int
    seq_lens: Tuple[int, ...]   # context tokens per sequence
    mix: Tuple[float, ...]      # P(FP16, INT4, INT2), or P(FP16, INT8, INT4, INT2); ignored if dirichlet
    num_layers: int = 1
    dirichlet: bool = False
    seed_offset: int = 0

    @property
    def num_chunks(self) -> Tuple[int, ...]:
        return tuple(t // self.chunk_size for t in self.seq_lens)


def _rng(*key: int) -> np.random.Generator:
    return np.random.default_rng([BASE_SEED, *[int(k) for k in key]])


def config(n: int) -> Workload:
    """The five benchmark configurations (1-based), and extra shapes for profiling from 6 on."""
    if n == 1:
        return Workload("cfg1_2k_8h", 1, 1, 8, 8, 128, 128, 32, (2048,), (0.1, 0.3, 0.6))
    if n == 2:
        return Workload("cfg2_llama2_7b_32k", 2, 1, 32, 32, 128, 256, 32, (32768,),
                        (0.1, 0.3, 0.6), num_layers=32)
    if n == 3:
        return Workload("cfg3_llama3_8b_gqa_64k_b4", 3, 4, 32, 8, 128, 256, 32,
                        (65536,) * 4, (0.15, 0.35, 0.5))
    if n == 4:
        return Workload("cfg4_llama2_13b_128k", 4, 1, 40, 40, 128, 512, 64, (131072,),
                        (0.05, 0.25, 0.7))
    if n == 5:
        r = _rng(5, _TAG_LEN)
        lens = tuple(int(x) * 256 for x in r.integers(8192 // 256, 131072 // 256 + 1, size=8))
        return Workload("cfg5_ragged_gqa_b8", 5, 8, 32, 8, 128, 256, 32, lens,
                        (1 / 3, 1 / 3, 1 / 3), dirichlet=True)
    if n == 6:
        # not one of the benchmark's five: a Llama-3-70B-shaped layer (8 query heads per kv head), the shape the
        # two-wave grouped-query kernel is profiled on
        return Workload("x6_gqa_64q_8kv_128k_b4", 6, 4, 64, 8, 128, 256, 32, (131072,) * 4, (0.15, 0.35, 0.5))
    if n == 7:
        # extra: head_dim 64 (64 heads of 64 channels, one query head per kv head), 128K context
        return Workload("x7_d64_64h_128k", 7, 1, 64, 64, 64, 256, 32, (131072,), (0.1, 0.3, 0.6))
    if n == 8:
        # extra: a four-class mix with INT8 chunks (FP16, INT8, INT4, INT2), 128K context, 32 heads
        return Workload("x8_int8_mix_32h_128k", 8, 1, 32, 32, 128, 256, 64, (131072,), (0.05, 0.15, 0.3, 0.5))
    if n == 9:
        # extra: the same four-class mix on a grouped-query shape
        return Workload("x9_int8_mix_gqa_64k_b4", 9, 4, 32, 8, 128, 256, 64, (65536,) * 4, (0.05, 0.15, 0.3, 0.5))
    raise ValueError(f"unknown config {n}")


def small(name: str, batch: int, hq: int, hkv: int, seq_lens: Sequence[int], chunk: int,
          group: int, mix=(0.2, 0.3, 0.5), head_dim: int = 128, seed_offset: int = 0) -> Workload:
    """An ad-hoc small workload for tests (config id 0)."""
    return Workload(name, 0, batch, hq, hkv, head_dim, chunk, group, tuple(int(t) for t in seq_lens),
                    tuple(mix), seed_offset=seed_offset)


def chunk_bits(w: Workload) -> List[np.ndarray]:
    """Per sequence: uint8 array [N_b] with values in {2, 4, 16} (and 8 where the mix has four entries)."""
    out = []
    for b, n in enumerate(w.num_chunks):
        r = _rng(w.config, w.seed_offset, b, _TAG_BITS)
        if w.dirichlet:
            if b == 0:
                p = np.array([1.0, 0.0, 0.0])
            elif b == 1:
                p = np.array([0.0, 0.0, 1.0])
            else:
                p = _rng(w.config, w.seed_offset, b, _TAG_MIX).dirichlet([1.0, 1.0, 1.0])
        else:
            p = np.asarray(w.mix, dtype=np.float64)
        p = p / p.sum()
        labels = [16, 4, 2] if len(p) == 3 else [16, 8, 4, 2]
        lab = r.choice(np.array(labels, dtype=np.uint8), size=n, p=p)
        out.append(lab.astype(np.uint8))
    return out


def outlier_channels(w: Workload, layer: int, h: int) -> np.ndarray:
    r = _rng(w.config, w.seed_offset, layer, h, _TAG_OUTLIER)
    return np.sort(r.choice(w.head_dim, size=4, replace=False))


def kv_head(w: Workload, layer: int, b: int, h: int) -> Tuple[np.ndarray, np.ndarray]:
    """K and V of one (sequence, kv-head): two fp16 arrays [T_b, D]."""
    t, d = w.seq_lens[b], w.head_dim
    k = _rng(w.config, w.seed_offset, layer, b, h, _TAG_K).standard_normal((t, d), dtype=np.float32)
    k[:, outlier_channels(w, layer, h)] *= np.float32(10.0)
    v = _rng(w.config, w.seed_offset, layer, b, h, _TAG_V).standard_normal((t, d), dtype=np.float32)
    return k.astype(np.float16), v.astype(np.float16)


def query(w: Workload, layer: int) -> np.ndarray:
    """q: fp16 [B, Hq, D]."""
    q = np.empty((w.batch, w.num_q_heads, w.head_dim), dtype=np.float16)
    for b in range(w.batch):
        for h in range(w.num_q_heads):
            q[b, h] = _rng(w.config, w.seed_offset, layer, b, h, _TAG_Q).standard_normal(
                w.head_dim, dtype=np.float32).astype(np.float16)
    return q


def seq_token_offsets(w: Workload) -> np.ndarray:
    """Token offset of each sequence in the flat ragged layout [sum T_b] (int64, [B+1])."""
    off = np.zeros(w.batch + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.asarray(w.seq_lens, dtype=np.int64))
    return off


def kv_flat(w: Workload, layer: int, threads: int = 8,
            out_k: Optional[np.ndarray] = None, out_v: Optional[np.ndarray] = None
            ) -> Tuple[np.ndarray, np.ndarray]:
    """All heads of a layer in one flat fp16 buffer each for K and V.

    Layout: sequence b starts at element seq_token_offsets[b] * Hkv * D; inside a
    sequence the order is [Hkv, T_b, D] (head-major), D contiguous.
    """
    off = seq_token_offsets(w)
    total = int(off[-1]) * w.num_kv_heads * w.head_dim
    k = out_k if out_k is not None else np.empty(total, dtype=np.float16)
    v = out_v if out_v is not None else np.empty(total, dtype=np.float16)
    assert k.size == total and v.size == total

    def fill(job):
        b, h = job
        t, d = w.seq_lens[b], w.head_dim
        base = (int(off[b]) * w.num_kv_heads + h * t) * d
        kk, vv = kv_head(w, layer, b, h)
        k[base:base + t * d] = kk.reshape(-1)
        v[base:base + t * d] = vv.reshape(-1)

    jobs = [(b, h) for b in range(w.batch) for h in range(w.num_kv_heads)]
    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    return k, v


def embeddings(name_seed: int, num_chunks: Sequence[int], embed_dim: int = 768,
               relevant_share: float = 0.08) -> Tuple[np.ndarray, List[np.ndarray]]:
    """Query and chunk embeddings for the chunk-level quantization search (Sec. III-B).

    Stand-ins for the encoder outputs (the paper uses a 768-wide retrieval encoder): Gaussian chunk
    embeddings of which a small share leans towards the query, the rest does not (Sec. I, Fig. 1: few
    chunks are relevant to a query).  Returns q fp32 [B, E] and per sequence c fp32 [N_b, E].
    """
    q = np.empty((len(num_chunks), embed_dim), dtype=np.float32)
    cs = []
    for b, n in enumerate(num_chunks):
        r = _rng(int(name_seed), b, _TAG_EMB)
        q[b] = r.standard_normal(embed_dim, dtype=np.float32)
        c = r.standard_normal((int(n), embed_dim), dtype=np.float32)
        lean = np.where(r.random(int(n)) < relevant_share, r.uniform(0.5, 2.0, int(n)), r.uniform(0.0, 0.3, int(n)))
        cs.append((c + lean[:, None].astype(np.float32) * q[b]).astype(np.float32))
    return q, cs
