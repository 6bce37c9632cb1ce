"""Pins for the oracle's base solution of Sec. 3.1 (migration, then de-fragmentation, into a
second pool), CPU only.  The merged cache is read back with helpers.page_in (numpy reshape /
transpose) and compared with the logical caches the source pools were paged out from, the
table with numpy cumsum, the counts with the input lengths, and one case with torch
indexing: none of it uses the oracle's own index arithmetic."""
import os

import numpy as np
import pytest
import torch

import oracle
from helpers import HEAD_MAJOR, TOKEN_MAJOR, logical_kv, page_in, page_out, random_table

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
SENT = 0xBEEF


def make(m, k, lens_per_inst, lay_s, lay_d, n_heads=8, d=4, B=4, layers=2, seed=0, slack=3):
    S = len(lens_per_inst[0])
    nb = [(np.asarray(l, dtype=np.int64) + B - 1) // B for l in lens_per_inst]
    P = int(max(x.sum() for x in nb)) + 4
    W = int(max(x.max(initial=0) for x in nb)) + 2
    insts = []
    for g in range(m):
        lens = np.asarray(lens_per_inst[g], dtype=np.int32)
        table = random_table(lens, B, P, seed=seed * 10 + g, width=W)
        kv = logical_kv(layers, lens, n_heads, d, np.uint16, seed=seed * 100 + g)
        pools = page_out(kv, lens, table, P, k, lay_s, B, filler_seed=seed + 50 + g)
        insts.append(dict(lens=lens, table=table, kv=kv, pools=pools, nb=nb[g]))
    total = int(sum(x.sum() for x in nb))
    cfg = oracle.KV(kv_layers=layers, n_kv_heads=n_heads, head_dim=d, block_tokens=B, num_seqs=S,
                    max_blocks_per_seq=W, src_pool_blocks=P, dst_pool_blocks=total + slack,
                    layout_src=lay_s, layout_dst=lay_d)
    return cfg, insts, total


def run_all_ranks(cfg, insts, m, k):
    out = {}
    be = cfg.n_kv_heads // (k * m) * 2 * cfg.block_tokens * cfg.head_dim
    for s in range(k):
        for g in range(m):
            fresh = np.full((cfg.kv_layers, cfg.dst_pool_blocks, be), SENT, dtype=np.uint16)
            pools = [insts[g2]["pools"][s] for g2 in range(m)]
            before = [p.copy() for p in pools]
            st, table, mig, dfr = oracle.merge_kv_base(cfg, k, m, s * m + g, pools,
                                                       [i["table"] for i in insts],
                                                       [i["lens"] for i in insts], fresh)
            assert st == oracle.OK
            for a, b in zip(pools, before):
                np.testing.assert_array_equal(a, b)          # the old pools are only read
            out[s * m + g] = (fresh, table, mig, dfr)
    return out


LENS = [[13, 1, 8, 0], [5, 22, 3, 9], [16, 2, 7, 7], [1, 1, 30, 4]]


@pytest.mark.parametrize("lay_s,lay_d", [(TOKEN_MAJOR, TOKEN_MAJOR), (HEAD_MAJOR, HEAD_MAJOR),
                                         (TOKEN_MAJOR, HEAD_MAJOR), (HEAD_MAJOR, TOKEN_MAJOR)])
@pytest.mark.parametrize("m,k", [(4, 1), (2, 1), (2, 2), (3, 2), (2, 4)])
def test_new_pools_read_back_as_the_union_of_all_requests(m, k, lay_s, lay_d):
    heads = 12 if k * m == 6 else k * m * 2
    cfg, insts, total = make(m, k, LENS[:m], lay_s, lay_d, n_heads=heads, seed=m * 3 + k)
    res = run_all_ranks(cfg, insts, m, k)
    tables = [res[r][1] for r in range(k * m)]
    for t in tables[1:]:
        np.testing.assert_array_equal(t, tables[0])           # one table serves every rank
    # compact ids over the merged sequence list, instance-major
    nb = np.concatenate([i["nb"] for i in insts])
    base = np.concatenate([[0], np.cumsum(nb)[:-1]])
    want = np.full_like(tables[0], -1)
    for row, (b, n) in enumerate(zip(base, nb)):
        want[row, :n] = np.arange(b, b + n)
    np.testing.assert_array_equal(tables[0], want)
    all_lens = np.concatenate([i["lens"] for i in insts])
    back = page_in([res[r][0] for r in range(k * m)], all_lens, tables[0], k * m, lay_d,
                   cfg.block_tokens, heads, cfg.head_dim)
    for l in range(cfg.kv_layers):
        for g in range(m):
            for i in range(cfg.num_seqs):
                np.testing.assert_array_equal(back[l][g * cfg.num_seqs + i], insts[g]["kv"][l][i])
    for r, (fresh, _, mig, dfr) in res.items():
        g = r % m
        assert dfr == int(insts[g]["nb"].sum())                # the local requests, compacted
        assert mig == total - dfr                              # everybody else's, received
        assert (fresh[:, total:] == SENT).all()                # blocks past the total untouched


def test_worked_example_heads_per_worker():
    """Sec. 3.1: H = 8, 4 x TP1 -> TP4: worker Wi ends up with heads 2i-1, 2i of every request
    (W2 retains H3, H4 and sends the rest away): the golden file."""
    want = {}
    for line in open(os.path.join(GOLDEN, "kv_head_ranges_H8_TP4.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w, heads = line.split(":")
        want[int(w.strip()[1:])] = sorted(int(h[1:]) for h in heads.split())
    m, k, H, d, B = 4, 1, 8, 2, 4
    cfg, insts, total = make(m, k, [[9, 4], [1, 12], [7, 7], [3, 16]], TOKEN_MAJOR, TOKEN_MAJOR,
                             n_heads=H, d=d, B=B, layers=1, seed=5)
    for inst in insts:                        # tag every element with its 1-based head
        for a in inst["kv"][0]:
            a[:] = np.arange(1, H + 1, dtype=np.uint16)[None, :, None, None]
        inst["pools"] = page_out(inst["kv"], inst["lens"], inst["table"], cfg.src_pool_blocks, k,
                                 TOKEN_MAJOR, B)
    res = run_all_ranks(cfg, insts, m, k)
    all_lens = np.concatenate([i["lens"] for i in insts])
    for worker in range(1, 5):
        fresh, table, _, _ = res[worker - 1]
        got = page_in([fresh], all_lens, table, 1, TOKEN_MAJOR, B, H // m, d)
        seen = sorted(set(np.concatenate([a.ravel() for a in got[0]]).tolist()))
        assert seen == want[worker]


def test_token_first_two_instances_reduce_to_torch_indexing():
    """m = 2, k = 1, token-first: new block = old block [K/V][token][heads g*H/2 ..][d], blocks
    of instance 0 first, then instance 1 (index_select + slicing)."""
    m, k = 2, 1
    cfg, insts, total = make(m, k, [[9, 16, 2], [5, 5, 11]], TOKEN_MAJOR, TOKEN_MAJOR, seed=8)
    res = run_all_ranks(cfg, insts, m, k)
    L, P, B, H, d = cfg.kv_layers, cfg.src_pool_blocks, cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim
    for g in range(m):
        got = torch.from_numpy(res[g][0].view(np.int16))[:, :total].reshape(L, total, 2, B, H // 2, d)
        parts = []
        for g2 in range(m):
            t = insts[g2]["table"]
            ids = torch.from_numpy(np.concatenate([t[i, :n] for i, n in enumerate(insts[g2]["nb"])])
                                   .astype(np.int64))
            old = torch.from_numpy(insts[g2]["pools"][0].view(np.int16)).view(L, P, 2, B, H, d)
            parts.append(old.index_select(1, ids)[..., g * (H // 2):(g + 1) * (H // 2), :])
        assert torch.equal(got, torch.cat(parts, dim=1))


def test_same_cache_as_the_in_place_merge():
    """Header-centric on both sides, the base solution and the in-place merge hold the same
    values under their own tables (different ids, same content)."""
    m, k = 4, 1
    cfg, insts, total = make(m, k, LENS, HEAD_MAJOR, HEAD_MAJOR, seed=2)
    res = run_all_ranks(cfg, insts, m, k)
    all_lens = np.concatenate([i["lens"] for i in insts])
    H, d, B = cfg.n_kv_heads, cfg.head_dim, cfg.block_tokens
    sub = H // m * 2 * B * d
    for g in range(m):
        local = insts[g]["pools"][0].copy()
        st, itable, _ = oracle.merge_kv_inplace(cfg, k, m, g, local,
                                                [None if g2 == g else insts[g2]["pools"][0]
                                                 for g2 in range(m)],
                                                [i["table"] for i in insts],
                                                [i["lens"] for i in insts])
        assert st == oracle.OK
        inplace = page_in([local.reshape(cfg.kv_layers, cfg.src_pool_blocks * m, sub)], all_lens,
                          itable, 1, HEAD_MAJOR, B, H // m, d)
        base = page_in([res[g][0]], all_lens, res[g][1], 1, HEAD_MAJOR, B, H // m, d)
        for l in range(cfg.kv_layers):
            for a, b in zip(inplace[l], base[l]):
                np.testing.assert_array_equal(a, b)


def test_errors():
    m, k = 2, 1
    cfg, insts, total = make(m, k, [[9, 4], [5, 8]], TOKEN_MAJOR, TOKEN_MAJOR, seed=3)
    tabs, lens = [i["table"] for i in insts], [i["lens"] for i in insts]
    pools = [i["pools"][0] for i in insts]
    be = oracle.kv_block_elems(cfg, 2)
    fresh = np.full((cfg.kv_layers, cfg.dst_pool_blocks, be), SENT, dtype=np.uint16)
    bad = [lens[0], lens[1].copy()]
    bad[1][0] = -2
    st, table, mig, dfr = oracle.merge_kv_base(cfg, k, m, 0, pools, tabs, bad, fresh)
    assert st == oracle.ERR_OVERFLOW and (table == -1).all() and mig == dfr == 0
    assert (fresh == SENT).all()
    long = [lens[0], lens[1].copy()]
    long[1][1] = (cfg.max_blocks_per_seq + 1) * cfg.block_tokens
    st, table, _, _ = oracle.merge_kv_base(cfg, k, m, 0, pools, tabs, long, fresh)
    assert st == oracle.ERR_OVERFLOW and (table == -1).all() and (fresh == SENT).all()
    import dataclasses
    small = dataclasses.replace(cfg, dst_pool_blocks=total - 1)
    st, table, _, _ = oracle.merge_kv_base(small, k, m, 0, pools, tabs, lens, fresh)
    assert st == oracle.ERR_OVERFLOW and (table == -1).all() and (fresh == SENT).all()
    bad_tab = [tabs[0], tabs[1].copy()]
    bad_tab[1][0, 1] = cfg.src_pool_blocks
    st, table, mig, dfr = oracle.merge_kv_base(cfg, k, m, 0, pools, bad_tab, lens, fresh)
    assert st == oracle.ERR_BLOCK_ID
    skipped = table[cfg.num_seqs, 1]
    assert skipped >= 0 and (fresh[:, skipped] == SENT).all()     # id assigned, block untouched
    assert mig == int(insts[1]["nb"].sum()) - 1 and dfr == int(insts[0]["nb"].sum())
    assert oracle.merge_kv_base(cfg, k, m, 2, pools, tabs, lens, fresh)[0] == oracle.ERR_ARG
    assert oracle.merge_kv_base(cfg, k, m, 0, [pools[0], None], tabs, lens, fresh)[0] == oracle.ERR_ARG
    assert oracle.merge_kv_base(cfg, k, 1, 0, pools[:1], tabs[:1], lens[:1], fresh)[0] == oracle.ERR_ARG
