"""Seeded synthetic inputs with the shapes and statistics of the paper's workloads.

This module serves both the GPU path's tests/benchmark and the CPU oracle.  It
holds no arithmetic of the method itself (no normalisation, projection,
softmax, MLP or merging): it only draws tensors.  Everything is numpy on the
host; the caller uploads what it needs.

The paper evaluates on Llama2-7B/13B/70B (Table 3: hidden sizes 4096 / 5120 /
8192, vocabulary 32000) with K = 4 speculative tokens and a 3K -> 512 -> 1
predictor (Sec. 4.3.2); neither weights nor datasets are needed here, only
those shapes.  Distributions: LM head ~ N(0, 0.02), RMSNorm weight
~ 1 + N(0, 0.01), hidden states ~ N(0, 1), predictor weights ~ N(0, 0.05),
all rounded to fp16.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


def _rng(seed, stream):
    return np.random.Generator(np.random.PCG64([int(seed), int(stream)]))


def lm_head(V: int, d: int, seed: int, std: float = 0.02, chunk_rows: int = 4096) -> np.ndarray:
    """[V][d] fp16, row v = output embedding of token v."""
    rng = _rng(seed, 1)
    out = np.empty((V, d), dtype=np.float16)
    for r0 in range(0, V, chunk_rows):
        r1 = min(V, r0 + chunk_rows)
        blk = rng.standard_normal((r1 - r0, d), dtype=np.float32)
        blk *= np.float32(std)
        out[r0:r1] = blk
    return out


def quantize_q4(w: np.ndarray, group: int = 128, chunk_rows: int = 2048):
    """4-bit group-quantised copy of an fp16 matrix [V][d], the storage the quantised-rows predictor reads:
    every run of `group` consecutive elements of a row gets an fp16 scale and an fp16 zero-point (an
    integer 0..15, the usual asymmetric min/max scheme) and each element a code 0..15.
    Returns (qweight uint32 [V][d/8], scales fp16 [V][d/group], zeros fp16 [V][d/group]); element i of a row
    sits in bits 4*(i%8) .. 4*(i%8)+3 of word i//8.  This only prepares inputs; how codes are turned back
    into weights is the business of the oracle and of the kernels, each on its own."""
    V, d = w.shape
    assert d % group == 0 and group % 8 == 0
    ng = d // group
    q = np.empty((V, d // 8), dtype=np.uint32)
    scales = np.empty((V, ng), dtype=np.float16)
    zeros = np.empty((V, ng), dtype=np.float16)
    shifts = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    for r0 in range(0, V, chunk_rows):
        blk = w[r0:r0 + chunk_rows].astype(np.float32).reshape(-1, ng, group)
        lo, hi = blk.min(axis=2), blk.max(axis=2)
        sc = np.maximum((hi - lo) / 15.0, 1e-8).astype(np.float16)          # what is stored is what is used
        sc32 = sc.astype(np.float32)
        zp = np.clip(np.rint(-lo / sc32), 0, 15)
        code = np.clip(np.rint(blk / sc32[:, :, None] + zp[:, :, None]), 0, 15).astype(np.uint32)
        words = (code.reshape(blk.shape[0], d // 8, 8) << shifts).sum(axis=2, dtype=np.uint32)
        q[r0:r0 + chunk_rows] = words
        scales[r0:r0 + chunk_rows] = sc
        zeros[r0:r0 + chunk_rows] = zp.astype(np.float16)
    return q, scales, zeros


def gamma(d: int, seed: int) -> np.ndarray:
    return (1.0 + 0.01 * _rng(seed, 2).standard_normal(d)).astype(np.float16)


def hidden(n: int, d: int, seed: int, lead=()) -> np.ndarray:
    return _rng(seed, 3).standard_normal(tuple(lead) + (n, d), dtype=np.float32).astype(np.float16)


def hidden_drift(L: int, B: int, d: int, seed: int, sigma: float = 0.1) -> np.ndarray:
    """[L][B][d]: h_0 ~ N(0,1), h_l = h_{l-1} + N(0, sigma), carried in fp32, rounded per layer."""
    rng = _rng(seed, 4)
    cur = rng.standard_normal((B, d), dtype=np.float32)
    out = np.empty((L, B, d), dtype=np.float16)
    for l in range(L):
        if l:
            cur = cur + np.float32(sigma) * rng.standard_normal((B, d), dtype=np.float32)
        out[l] = cur
    return out


def ids_uniform_distinct(B: int, K: int, V: int, seed: int) -> np.ndarray:
    rng = _rng(seed, 5)
    return np.stack([rng.choice(V, size=K, replace=False) for _ in range(B)]).astype(np.int32)


def _zipf_p(n: int, a: float) -> np.ndarray:
    p = np.arange(1, n + 1, dtype=np.float64) ** (-a)
    return p / p.sum()


def ids_zipf_pool(N: int, K: int, V: int, pool: int, seed: int, a: float = 1.1) -> np.ndarray:
    """Per node K distinct ids drawn by Zipf(a) rank from a pool of `pool` distinct
    uniform token ids, so that the union over the N nodes is at most `pool`."""
    rng = _rng(seed, 6)
    pool_ids = rng.choice(V, size=pool, replace=False)
    p = _zipf_p(pool, a)
    return np.stack([pool_ids[rng.choice(pool, size=K, replace=False, p=p)] for _ in range(N)]).astype(np.int32)


def ids_zipf_vocab(B: int, K: int, V: int, seed: int, a: float = 1.1) -> np.ndarray:
    """Per sequence K distinct ids, Zipf(a) rank over the whole vocabulary mapped
    through a fixed seeded permutation of the vocabulary."""
    rng = _rng(seed, 7)
    perm = rng.permutation(V)
    p = _zipf_p(V, a)
    return np.stack([perm[rng.choice(V, size=K, replace=False, p=p)] for _ in range(B)]).astype(np.int32)


def prob_rows(shape, K: int, seed: int) -> np.ndarray:
    """Valid probability vectors (flat Dirichlet) standing in for the previous layer's local probabilities."""
    return _rng(seed, 8).dirichlet(np.ones(K), size=shape).astype(np.float32)


def mlp(K: int, H: int, seed: int, L: int | None = None, bias: bool = False, std: float = 0.05):
    """Predictor weights: W1 [H][3K] (output x input), w2 [H]; optional b1 [H], b2 [1].
    With L given, one predictor per layer: leading dimension L on every array."""
    rng = _rng(seed, 9)
    lead = () if L is None else (L,)
    W1 = (std * rng.standard_normal(lead + (H, 3 * K))).astype(np.float16)
    w2 = (std * rng.standard_normal(lead + (H,))).astype(np.float16)
    b1 = b2 = None
    if bias:
        b1 = (std * rng.standard_normal(lead + (H,))).astype(np.float16)
        b2 = (std * rng.standard_normal(lead + (1,) if L is None else lead)).astype(np.float16)
    return dict(W1=W1, w2=w2, b1=b1, b2=b2)


def tree_parents(widths, seed: int, max_children: int = 4) -> np.ndarray:
    """Level-by-level tree: level 0 nodes are roots (-1); each later node picks a parent
    uniformly among previous-level nodes that still have fewer than max_children."""
    rng = _rng(seed, 10)
    parent = []
    prev_level = []
    for lvl, w in enumerate(widths):
        start = len(parent)
        if lvl == 0:
            parent += [-1] * w
        else:
            kids = {p: 0 for p in prev_level}
            for _ in range(w):
                free = [p for p in prev_level if kids[p] < max_children]
                p = int(free[rng.integers(len(free))])
                kids[p] += 1
                parent.append(p)
        prev_level = list(range(start, start + w))
    return np.asarray(parent, dtype=np.int32)


@dataclass(frozen=True)
class Config:
    name: str
    d: int
    V: int
    K: int
    H: int = 512
    L: int = 1          # layers (sweep configs)
    B: int = 1          # independent tokens / sequences
    N: int = 0          # tree nodes (0 = not a tree config)
    Mcap: int = 0       # bound on the merged set
    widths: tuple = ()
    eps: float = 1e-5
    threshold: float = 0.5
    note: str = ""


CONFIGS = {
    # the five workloads of the benchmark definition
    "C1": Config("C1", d=4096, V=32000, K=4, note="single predictor step, Llama2-7B shape"),
    "C2": Config("C2", d=4096, V=32000, K=4, L=32, note="32-layer exit sweep for one token"),
    "C3": Config("C3", d=4096, V=32000, K=4, N=60, Mcap=64, widths=(4, 8, 12, 14, 12, 10),
                 note="merged tree mapping, 60-node EAGLE-like tree"),
    "C4": Config("C4", d=5120, V=32000, K=4, L=40, B=16, note="Llama2-13B shape, 16 sequences x 40 layers"),
    "C5": Config("C5", d=8192, V=128256, K=8, N=64, Mcap=256, widths=(4, 8, 12, 14, 14, 12),
                 note="large-vocabulary tree stress"),
    # small shapes for exhaustive parity: several tiles plus ragged tails
    "T1": Config("T1", d=64, V=50, K=3, H=40, B=5),
    "T2": Config("T2", d=1032, V=301, K=4, H=512, B=7, L=5),
    "T3": Config("T3", d=2056, V=997, K=5, H=200, N=37, Mcap=96, widths=(3, 6, 9, 10, 9)),
    "T4": Config("T4", d=520, V=777, K=8, H=512, N=21, Mcap=168, widths=(2, 4, 7, 8)),
}


def make(name: str, seed: int = 0, bias: bool = False, lm=None) -> dict:
    """All host tensors of one configuration.  `lm` lets callers share one LM head
    between configurations of the same (V, d) (it is by far the largest draw)."""
    c = CONFIGS[name] if isinstance(name, str) else name
    idx = sorted(CONFIGS).index(c.name) if c.name in CONFIGS else 99
    s = 1000 * (idx + 1) + seed
    out = dict(cfg=c)
    out["lm_head"] = lm if lm is not None else lm_head(c.V, c.d, lm_seed(c))
    out["gamma"] = gamma(c.d, s)
    if c.N:  # tree
        assert sum(c.widths) == c.N
        out["hidden"] = hidden(c.N, c.d, s)
        out["parent"] = tree_parents(c.widths, s)
        pool = min(c.Mcap, c.V)
        out["ids"] = ids_zipf_pool(c.N, c.K, c.V, pool, s)
        out["prev_probs"] = prob_rows(c.N, c.K, s)
        out.update(mlp(c.K, c.H, s, bias=bias))
    elif c.L > 1:  # sweep
        if c.B == 1:
            out["hidden"] = hidden_drift(c.L, c.B, c.d, s)
            out["ids"] = ids_uniform_distinct(c.B, c.K, c.V, s)
        else:
            out["hidden"] = hidden(c.B, c.d, s, lead=(c.L,))
            out["ids"] = ids_zipf_vocab(c.B, c.K, c.V, s)
        out.update(mlp(c.K, c.H, s, L=c.L, bias=bias))
    else:
        out["hidden"] = hidden(c.B, c.d, s)
        out["ids"] = ids_uniform_distinct(c.B, c.K, c.V, s)
        out["prev_probs"] = prob_rows(c.B, c.K, s)
        out.update(mlp(c.K, c.H, s, bias=bias))
    return out


def lm_seed(c: Config) -> int:
    """LM heads depend on the shape only, so configurations of one model share them."""
    return 7_000_000 + c.V * 16 + c.d
