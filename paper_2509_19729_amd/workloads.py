"""Seeded synthetic inputs shared by the oracle tests, the GPU parity tests and bench.py.

This module only *draws inputs*: model shapes, sequence lengths, paged block
placements and opaque 16-bit payloads.  It contains none of the reshard
arithmetic (no head ranges, no shard offsets, no layout indexing) so that the
CPU oracle and the HIP library stay independent of each other.

The five workloads mirror the configurations the benchmark is defined on
(tiny decoder, 7B-, 13B-, 70B-GQA- and long-context 8B-shaped).  The paper's
own workload is a private production trace (Sec. 2.3, Sec. 4.3); these stand in
for it.  Choices the configuration text leaves open (lognormal sigma = 1, a
32K cap on the Pareto tail, pool slack of 5 %) are made here.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

HEAD_MAJOR = 0
TOKEN_MAJOR = 1


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                # 1..5, also the seed of the length / placement draws
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    dtype: str                # "fp16" | "bf16" (payload is opaque 16-bit either way)
    src_tp: int
    dst_tp: int
    dst_rank: int
    block_tokens: int
    num_seqs: int
    lengths: str              # recipe name, see seq_lens()
    placement: str            # recipe name, see block_placement()
    elem_bytes: int = 2
    n_experts: int = 0        # > 0: mixture of experts, ffn_dim is one expert's intermediate size

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    "tiny": Workload("tiny", 1, 2, 256, 8, 8, 32, 1024, "fp16", 1, 2, 0, 16, 4,
                     "uniform_1_512", "perm128"),
    "llama7b": Workload("llama7b", 2, 32, 4096, 32, 32, 128, 11008, "bf16", 4, 2, 1, 16, 64,
                        "lognormal_1k_8k", "freelist_rr"),
    "llama13b": Workload("llama13b", 3, 40, 5120, 40, 40, 128, 13824, "bf16", 2, 1, 0, 16, 128,
                         "uniform_128_4096", "fragmented80"),
    "gqa70b": Workload("gqa70b", 4, 80, 8192, 64, 8, 128, 28672, "bf16", 8, 4, 2, 16, 32,
                       "lognormal_2k_16k", "freelist_rr"),
    "long8b": Workload("long8b", 5, 32, 4096, 32, 8, 128, 14336, "bf16", 1, 4, 3, 16, 64,
                       "long32k_pareto", "random105"),
    # outside the five benchmark configurations: the mixture-of-experts shape of the paper's
    # EP experiment (Sec. 4.3, 4 x (TP1 EP1) -> TP4 EP4), 128 experts of 768 x 2048
    "qwen3moe": Workload("qwen3moe", 6, 48, 2048, 32, 4, 128, 768, "bf16", 1, 4, 1, 16, 64,
                         "lognormal_1k_8k", "freelist_rr", n_experts=128),
}
ORDER = ["tiny", "llama7b", "llama13b", "gqa70b", "long8b"]


def seq_lens(w: Workload) -> np.ndarray:
    """Sequence lengths in tokens, int32 [num_seqs], seeded by the workload index."""
    rng = np.random.default_rng(w.index)
    S = w.num_seqs
    if w.lengths == "uniform_1_512":
        out = rng.integers(1, 513, size=S)
    elif w.lengths == "lognormal_1k_8k":
        out = np.clip(np.round(1024.0 * np.exp(rng.standard_normal(S))), 1, 8192)
    elif w.lengths == "uniform_128_4096":
        out = rng.integers(128, 4097, size=S)
    elif w.lengths == "lognormal_2k_16k":
        out = np.clip(np.round(2048.0 * np.exp(rng.standard_normal(S))), 1, 16384)
    elif w.lengths == "long32k_pareto":
        n_long = min(8, S)
        u = rng.random(S - n_long)
        tail = np.minimum(np.floor(256.0 * (1.0 - u) ** (-1.0 / 1.5)), 32768)
        out = np.concatenate([np.full(n_long, 32768.0), tail])
    else:
        raise ValueError(w.lengths)
    return out.astype(np.int32)


def blocks_per_seq(lens: np.ndarray, block_tokens: int) -> np.ndarray:
    """Blocks a paged cache holds for each sequence (a property of the input structure)."""
    return (lens.astype(np.int64) + block_tokens - 1) // block_tokens


def block_placement(w: Workload, lens: np.ndarray):
    """Draw the source block table.  Returns (table int32 [S, W] padded with -1, src_pool_blocks)."""
    rng = np.random.default_rng(1000 + w.index)
    nb = blocks_per_seq(lens, w.block_tokens)
    need = int(nb.sum())
    W = max(8, int(-(-int(nb.max(initial=0)) // 8) * 8))
    table = np.full((len(lens), W), -1, dtype=np.int32)
    if w.placement == "perm128":
        pool = max(128, need)
        ids = rng.permutation(pool)[:need]
        order = "seq"
    elif w.placement == "freelist_rr":
        pool = int(np.ceil(need * 1.05))
        ids = rng.permutation(pool)[:need]
        order = "rr"
    elif w.placement == "fragmented80":
        pool = int(np.ceil(need / 0.8))
        ids = rng.permutation(pool)[:need]
        order = "seq"
    elif w.placement == "random105":
        pool = int(np.ceil(need * 1.05))
        ids = rng.permutation(pool)[:need]
        order = "seq"
    else:
        raise ValueError(w.placement)
    if order == "seq":
        p = 0
        for i, n in enumerate(nb):
            table[i, :n] = ids[p:p + n]
            p += int(n)
    else:
        # sequences grow together: the free list is popped round-robin, one block per
        # still-growing sequence per round
        p = 0
        for j in range(int(nb.max(initial=0))):
            alive = np.nonzero(nb > j)[0]
            table[alive, j] = ids[p:p + len(alive)]
            p += len(alive)
    return table, pool


def payload16(n: int, seed: int, dtype: str = "bf16") -> np.ndarray:
    """n opaque 16-bit patterns of values ~ N(0, 0.02) in bf16 (truncated) or fp16."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)
    if dtype == "fp16":
        return x.astype(np.float16).view(np.uint16)
    return (x.view(np.uint32) >> 16).astype(np.uint16)


def random_bits(n: int, seed: int, elem_bytes: int = 2) -> np.ndarray:
    """n uniformly random opaque elements (every bit pattern equally likely)."""
    rng = np.random.default_rng(seed)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32}[elem_bytes]
    return rng.integers(0, np.iinfo(dt).max, size=n, dtype=dt, endpoint=True)
