"""Test-side statement of the expert-wise shard of a mixture-of-experts decoder, in numpy
split / slicing / concatenate only (nothing here is imported by the oracle or the library).

Attention tensors are cut by head with ``np.split`` as for a dense model; rank r at degree t
keeps the whole experts ``experts[r*E/t:(r+1)*E/t]`` (Sec. 3.2, EP discussion), each stored as
gate, up, down one after the other; with ``page_elems`` > 0 the attention part and every expert
are padded with zeros to a multiple of it.
"""
from __future__ import annotations

import numpy as np


def moe_full_model(m, n_experts, seed=0, unique=False):
    """Per layer: dict with unsharded q, k, v, o and a list of (gate, up, down) per expert."""
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32}[m.elem_bytes]
    rng = np.random.default_rng(seed)
    H, d, f = m.hidden, m.head_dim, m.ffn_dim
    counter = [0]

    def fill(shape):
        n = int(np.prod(shape))
        if unique:
            assert m.elem_bytes == 4
            a = np.arange(counter[0], counter[0] + n, dtype=np.uint32).reshape(shape)
            counter[0] += n
            return a
        return rng.integers(0, np.iinfo(dt).max, size=shape, dtype=dt, endpoint=True)

    layers = []
    for _ in range(m.n_layers):
        L = {"q": fill((m.n_q_heads * d, H)), "k": fill((m.n_kv_heads * d, H)),
             "v": fill((m.n_kv_heads * d, H)), "o": fill((H, m.n_q_heads * d))}
        L["experts"] = [(fill((f, H)), fill((f, H)), fill((H, f))) for _ in range(n_experts)]
        layers.append(L)
    return layers


def _pad(flat, page_elems):
    flat = np.ascontiguousarray(flat).ravel()
    if page_elems <= 1:
        return flat
    n = -(-flat.size // page_elems) * page_elems
    return np.concatenate([flat, np.zeros(n - flat.size, dtype=flat.dtype)])


def moe_shard_of(layers, tp, rank, n_experts, page_elems=0):
    """Rank `rank`'s shard at degree tp (attention TP, experts EP)."""
    own = n_experts // tp
    parts = []
    for L in layers:
        attn = [np.split(L["q"], tp, axis=0)[rank], np.split(L["k"], tp, axis=0)[rank],
                np.split(L["v"], tp, axis=0)[rank],
                np.ascontiguousarray(np.split(L["o"], tp, axis=1)[rank])]
        parts.append(_pad(np.concatenate([a.ravel() for a in attn]), page_elems))
        for g, u, dn in L["experts"][rank * own:(rank + 1) * own]:
            parts.append(_pad(np.concatenate([g.ravel(), u.ravel(), dn.ravel()]), page_elems))
    return np.concatenate(parts)
