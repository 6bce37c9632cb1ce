"""Test-side reference structures, written with numpy split / reshape / transpose only.

Nothing here is imported by the oracle or by the HIP library.  The helpers give
the tests a second, independent statement of the problem:

* an *unsharded* decoder (per-layer Wq, Wk, Wv, Wo, Wg, Wu, Wd, row-major
  [out, in]) cut into TP shards with ``np.split`` (Sec. 2.2 and Sec. 3.2 of the
  paper: heads / FFN segments spread evenly, up_proj by stored rows, down_proj
  by stored columns);
* a *logical* KV cache ``[layer][seq] -> array[token, head, K/V, d]`` paged into
  block pools with ``reshape``/``transpose`` for either block layout of Sec. 3.1,
  and read back the same way.
"""
from __future__ import annotations

import numpy as np

HEAD_MAJOR = 0
TOKEN_MAJOR = 1

TENSORS = ("q", "k", "v", "o", "g", "u", "d")


# ----------------------------------------------------------------------------- weights
def full_model(m, seed=0, unique=False):
    """List (per layer) of dicts of unsharded tensors filled with opaque elements."""
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32}[m.elem_bytes]
    rng = np.random.default_rng(seed)
    H, d = m.hidden, m.head_dim
    shapes = {"q": (m.n_q_heads * d, H), "k": (m.n_kv_heads * d, H), "v": (m.n_kv_heads * d, H),
              "o": (H, m.n_q_heads * d), "g": (m.ffn_dim, H), "u": (m.ffn_dim, H),
              "d": (H, m.ffn_dim)}
    layers, counter = [], 0
    for _ in range(m.n_layers):
        L = {}
        for name in TENSORS:
            n = shapes[name][0] * shapes[name][1]
            if unique:  # every element of the whole model gets its own value
                assert m.elem_bytes == 4
                L[name] = np.arange(counter, counter + n, dtype=np.uint32).reshape(shapes[name])
                counter += n
            else:
                L[name] = rng.integers(0, np.iinfo(dt).max, size=shapes[name], dtype=dt,
                                       endpoint=True)
        layers.append(L)
    return layers


def shard_of(layers, tp, rank):
    """Rank `rank`'s packed shard at TP=tp, by np.split on the unsharded tensors."""
    parts = []
    for L in layers:
        q = np.split(L["q"], tp, axis=0)[rank]
        k = np.split(L["k"], tp, axis=0)[rank]
        v = np.split(L["v"], tp, axis=0)[rank]
        o = np.split(L["o"], tp, axis=1)[rank]
        g = np.split(L["g"], tp, axis=0)[rank]
        u = np.split(L["u"], tp, axis=0)[rank]
        dn = np.split(L["d"], tp, axis=1)[rank]
        parts += [q.ravel(), k.ravel(), v.ravel(), np.ascontiguousarray(o).ravel(), g.ravel(),
                  u.ravel(), np.ascontiguousarray(dn).ravel()]
    return np.concatenate(parts)


def unpack_shard(shard, m, tp):
    """Inverse of the packing in shard_of: list (per layer) of dicts of the rank's tensors."""
    H, d = m.hidden, m.head_dim
    shapes = [("q", (m.n_q_heads * d // tp, H)), ("k", (m.n_kv_heads * d // tp, H)),
              ("v", (m.n_kv_heads * d // tp, H)), ("o", (H, m.n_q_heads * d // tp)),
              ("g", (m.ffn_dim // tp, H)), ("u", (m.ffn_dim // tp, H)),
              ("d", (H, m.ffn_dim // tp))]
    out, p = [], 0
    for _ in range(m.n_layers):
        L = {}
        for name, shp in shapes:
            n = shp[0] * shp[1]
            L[name] = shard[p:p + n].reshape(shp)
            p += n
        out.append(L)
    assert p == shard.size
    return out


def reassemble(shards, m, tp):
    """Concatenate all tp unpacked shards back into unsharded tensors."""
    un = [unpack_shard(s, m, tp) for s in shards]
    layers = []
    for l in range(m.n_layers):
        L = {}
        for name in TENSORS:
            axis = 1 if name in ("o", "d") else 0
            L[name] = np.concatenate([un[r][l][name] for r in range(tp)], axis=axis)
        layers.append(L)
    return layers


# ----------------------------------------------------------------------------- KV cache
def logical_kv(n_layers, lens, n_heads, d, dtype, seed=0, unique=False):
    """kv[l][i] = array [len_i, n_heads, 2, d] of opaque elements."""
    rng = np.random.default_rng(seed)
    out, counter = [], 0
    for _ in range(n_layers):
        row = []
        for n in lens:
            shp = (int(n), n_heads, 2, d)
            cnt = int(np.prod(shp))
            if unique:
                a = np.arange(counter, counter + cnt, dtype=np.uint32).astype(dtype).reshape(shp)
                counter += cnt
            else:
                a = rng.integers(0, np.iinfo(dtype).max, size=shp, dtype=dtype, endpoint=True)
            row.append(a)
        out.append(row)
    return out


def _block_view(flat_block, layout, heads, B, d):
    """View one block as [token, head, K/V, d] regardless of its storage order."""
    if layout == HEAD_MAJOR:       # stored [head][K/V][token][d]
        return flat_block.reshape(heads, 2, B, d).transpose(2, 0, 1, 3)
    return flat_block.reshape(2, B, heads, d).transpose(1, 2, 0, 3)  # stored [K/V][token][head][d]


def page_out(kv, lens, table, pool_blocks, tp, layout, B, filler_seed=99):
    """Write the logical cache into tp block pools [layers, pool_blocks, block_elems].

    Unused pool blocks and the slots past a sequence's end get random filler."""
    n_layers = len(kv)
    n_heads, d = kv[0][0].shape[1], kv[0][0].shape[3]
    dtype = kv[0][0].dtype
    hl = n_heads // tp
    rng = np.random.default_rng(filler_seed)
    pools = []
    for r in range(tp):
        pool = rng.integers(0, np.iinfo(dtype).max, size=(n_layers, pool_blocks, hl * 2 * B * d),
                            dtype=dtype, endpoint=True)
        for l in range(n_layers):
            for i, n in enumerate(lens):
                mine = kv[l][i][:, r * hl:(r + 1) * hl]      # heads this rank owns
                for j in range((int(n) + B - 1) // B):
                    view = _block_view(pool[l, table[i, j]], layout, hl, B, d)
                    chunk = mine[j * B:(j + 1) * B]
                    view[:chunk.shape[0]] = chunk
        pools.append(pool)
    return pools


def page_in(pools, lens, table, tp, layout, B, n_heads, d):
    """Read the logical cache back through a block table: kv[l][i] = [len_i, n_heads, 2, d]."""
    n_layers = pools[0].shape[0]
    hl = n_heads // tp
    out = []
    for l in range(n_layers):
        row = []
        for i, n in enumerate(lens):
            a = np.zeros((int(n), n_heads, 2, d), dtype=pools[0].dtype)
            for j in range((int(n) + B - 1) // B):
                lo, hi = j * B, min((j + 1) * B, int(n))
                for r in range(tp):
                    view = _block_view(pools[r][l, table[i, j]], layout, hl, B, d)
                    a[lo:hi, r * hl:(r + 1) * hl] = view[:hi - lo]
            row.append(a)
        out.append(row)
    return out


def random_table(lens, B, pool_blocks, seed=0, width=None):
    nb = (np.asarray(lens, dtype=np.int64) + B - 1) // B
    rng = np.random.default_rng(seed)
    ids = rng.permutation(pool_blocks)[:int(nb.sum())]
    W = width if width is not None else max(1, int(nb.max(initial=0))) + 2
    table = np.full((len(lens), W), -1, dtype=np.int32)
    p = 0
    for i, n in enumerate(nb):
        table[i, :n] = ids[p:p + n]
        p += int(n)
    return table
