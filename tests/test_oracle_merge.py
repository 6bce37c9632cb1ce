"""Pins for the oracle's in-place instance merge (Sec. 3.1, Improvement 1), CPU only.

m instances at TP=k, each with its own sequences and block table, become one instance
at TP=k*m.  The checks read the merged cache back with helpers.page_in (numpy
reshape/transpose) and compare with the logical caches the source pools were paged
out from, so they do not depend on the oracle's index arithmetic.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from helpers import HEAD_MAJOR, logical_kv, page_in, page_out, random_table

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make_instances(m, k, lens_per_inst, n_heads=8, d=4, B=4, layers=2, P=None, seed=0, W=None):
    """m instances at TP=k: logical caches, tables and per-rank pools (header-centric)."""
    S = len(lens_per_inst[0])
    nb = [(np.asarray(l, dtype=np.int64) + B - 1) // B for l in lens_per_inst]
    P = P or int(max(x.sum() for x in nb)) + 4
    W = W or int(max(x.max(initial=0) for x in nb)) + 2
    insts = []
    for g in range(m):
        lens = np.asarray(lens_per_inst[g], dtype=np.int32)
        table = random_table(lens, B, P, seed=seed * 10 + g, width=W)
        kv = logical_kv(layers, lens, n_heads, d, np.uint16, seed=seed * 100 + g)
        pools = page_out(kv, lens, table, P, k, HEAD_MAJOR, B, filler_seed=seed + 50 + g)
        insts.append(dict(lens=lens, table=table, kv=kv, pools=pools))
    cfg = oracle.KV(kv_layers=layers, n_kv_heads=n_heads, head_dim=d, block_tokens=B, num_seqs=S,
                    max_blocks_per_seq=W, src_pool_blocks=P, dst_pool_blocks=P * m)
    return cfg, insts


def merge_all_ranks(cfg, insts, m, k):
    """Run the oracle for every target rank r' = s*m + g on a private copy of its local pool."""
    out = {}
    for s in range(k):
        for g in range(m):
            local = insts[g]["pools"][s].copy()
            remote = [None if g2 == g else insts[g2]["pools"][s] for g2 in range(m)]
            st, table, n = oracle.merge_kv_inplace(cfg, k, m, s * m + g, local, remote,
                                                   [i["table"] for i in insts],
                                                   [i["lens"] for i in insts])
            assert st == oracle.OK
            out[s * m + g] = (local, table, n)
    return out


@pytest.mark.parametrize("m,k", [(4, 1), (2, 1), (2, 2), (3, 2), (2, 4)])
def test_merged_cache_reads_back_as_the_union_of_all_requests(m, k):
    lens = [[13, 1, 8, 0], [5, 22, 3, 9], [16, 2, 7, 7], [1, 1, 30, 4]][:m]
    cfg, insts = make_instances(m, k, lens, n_heads=k * m * 2 if (k * m) not in (6,) else 12,
                                seed=m * 3 + k)
    res = merge_all_ranks(cfg, insts, m, k)
    tables = [res[r][1] for r in range(k * m)]
    for t in tables[1:]:
        np.testing.assert_array_equal(t, tables[0])     # one table serves every rank
    H, d, B = cfg.n_kv_heads, cfg.head_dim, cfg.block_tokens
    sub = H // (k * m) * 2 * B * d
    new_pools = [res[r][0].reshape(cfg.kv_layers, cfg.src_pool_blocks * m, sub)
                 for r in range(k * m)]
    all_lens = np.concatenate([i["lens"] for i in insts])
    back = page_in(new_pools, all_lens, tables[0], k * m, HEAD_MAJOR, B, H, d)
    for l in range(cfg.kv_layers):
        for g in range(m):
            for i in range(cfg.num_seqs):
                np.testing.assert_array_equal(back[l][g * cfg.num_seqs + i], insts[g]["kv"][l][i])


def test_ids_are_reshaped_ids_and_local_heads_do_not_move():
    m, k = 4, 1
    lens = [[13, 1, 8, 0], [5, 22, 3, 9], [16, 2, 7, 7], [1, 1, 30, 4]]
    cfg, insts = make_instances(m, k, lens, seed=2)
    res = merge_all_ranks(cfg, insts, m, k)
    S, W, P, B = cfg.num_seqs, cfg.max_blocks_per_seq, cfg.src_pool_blocks, cfg.block_tokens
    table = res[0][1]
    for g in range(m):
        old = insts[g]["table"]
        want = np.where(old >= 0, old * m + g, -1)
        np.testing.assert_array_equal(table[g * S:(g + 1) * S], want)
    used = table[table >= 0]
    assert len(set(used.tolist())) == len(used) and used.max() < P * m
    sub = cfg.n_kv_heads // m * 2 * B * cfg.head_dim
    for g in range(m):
        local, _, n_remote = res[g]
        before = insts[g]["pools"][0].reshape(cfg.kv_layers, P * m, sub)
        after = local.reshape(cfg.kv_layers, P * m, sub)
        written = np.zeros(P * m, dtype=bool)
        for g2 in range(m):
            if g2 != g:
                ids = table[g2 * S:(g2 + 1) * S]
                written[ids[ids >= 0]] = True
        assert written.sum() == n_remote == sum(
            int(((insts[g2]["lens"].astype(np.int64) + B - 1) // B).sum())
            for g2 in range(m) if g2 != g)
        # everything that is not a received block is byte-identical: in place, no extra memory
        np.testing.assert_array_equal(after[:, ~written], before[:, ~written])
        # and the received blocks are the sender's sub-block g
        for g2 in range(m):
            if g2 == g:
                continue
            src = insts[g2]["pools"][0].reshape(cfg.kv_layers, P, m, sub)
            old = insts[g2]["table"]
            for b in old[old >= 0]:
                np.testing.assert_array_equal(after[:, b * m + g2], src[:, b, g])


def test_worked_example_4xTP1_to_TP4_heads_per_worker():
    """Sec. 3.1: H = 8, 4 x TP1 -> TP4.  W2 retains H3,H4 of its local requests and receives
    H3,H4 of everybody else's; in general Wi ends up with the heads the golden file lists."""
    want = {}
    for line in open(os.path.join(GOLDEN, "kv_head_ranges_H8_TP4.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w, heads = line.split(":")
        want[int(w.strip()[1:])] = sorted(int(h[1:]) for h in heads.split())
    m, k, H, d, B = 4, 1, 8, 2, 4
    lens = [[9, 4], [1, 12], [7, 7], [3, 16]]
    cfg, insts = make_instances(m, k, lens, n_heads=H, d=d, B=B, layers=1, seed=5)
    for inst in insts:                       # tag every element with its 1-based head
        for a in inst["kv"][0]:
            a[:] = np.arange(1, H + 1, dtype=np.uint16)[None, :, None, None]
        inst["pools"] = page_out(inst["kv"], inst["lens"], inst["table"], cfg.src_pool_blocks, k,
                                 HEAD_MAJOR, B)
    res = merge_all_ranks(cfg, insts, m, k)
    all_lens = np.concatenate([i["lens"] for i in insts])
    sub = H // m * 2 * B * d
    for worker in range(1, 5):
        local, table, _ = res[worker - 1]
        pool = local.reshape(1, cfg.src_pool_blocks * m, sub)
        got = page_in([pool], all_lens, table, 1, HEAD_MAJOR, B, H // m, d)
        seen = sorted(set(np.concatenate([a.ravel() for a in got[0]]).tolist()))
        assert seen == want[worker]


def test_two_instances_reduce_to_torch_indexing():
    m, k = 2, 1
    cfg, insts = make_instances(m, k, [[9, 16, 2], [5, 5, 11]], seed=8)
    res = merge_all_ranks(cfg, insts, m, k)
    P, L = cfg.src_pool_blocks, cfg.kv_layers
    for g in range(m):
        other = 1 - g
        ids = insts[other]["table"]
        ids = torch.from_numpy(ids[ids >= 0].astype(np.int64))
        got = torch.from_numpy(res[g][0].view(np.int16)).view(L, P, m, -1)
        src = torch.from_numpy(insts[other]["pools"][0].view(np.int16)).view(L, P, m, -1)
        assert torch.equal(got[:, ids, other], src[:, ids, g])
        mine = insts[g]["table"]
        mine = torch.from_numpy(mine[mine >= 0].astype(np.int64))
        orig = torch.from_numpy(insts[g]["pools"][0].view(np.int16)).view(L, P, m, -1)
        assert torch.equal(got[:, mine, g], orig[:, mine, g])


def test_errors():
    m, k = 2, 1
    cfg, insts = make_instances(m, k, [[9, 4], [5, 8]], seed=3)
    tabs, lens = [i["table"] for i in insts], [i["lens"] for i in insts]
    local = insts[0]["pools"][0].copy()
    bad = [lens[0], lens[1].copy()]
    bad[1][0] = -2
    st, table, n = oracle.merge_kv_inplace(cfg, k, m, 0, local, [None, insts[1]["pools"][0]], tabs,
                                           bad)
    assert st == oracle.ERR_OVERFLOW and (table == -1).all() and n == 0
    np.testing.assert_array_equal(local, insts[0]["pools"][0])
    long = [lens[0], lens[1].copy()]
    long[1][1] = (cfg.max_blocks_per_seq + 1) * cfg.block_tokens
    st, table, _ = oracle.merge_kv_inplace(cfg, k, m, 0, local, [None, insts[1]["pools"][0]],
                                           tabs, long)
    assert st == oracle.ERR_OVERFLOW and (table == -1).all()
    np.testing.assert_array_equal(local, insts[0]["pools"][0])
    bad_tab = [tabs[0], tabs[1].copy()]
    bad_tab[1][0, 1] = cfg.src_pool_blocks
    st, table, n = oracle.merge_kv_inplace(cfg, k, m, 0, local, [None, insts[1]["pools"][0]],
                                           bad_tab, lens)
    assert st == oracle.ERR_BLOCK_ID and table[cfg.num_seqs, 1] == -1
    assert oracle.merge_kv_inplace(cfg, k, m, 2, local, [None, insts[1]["pools"][0]], tabs,
                                   lens)[0] == oracle.ERR_ARG
    assert oracle.merge_kv_inplace(cfg, k, m, 0, local, [None, None], tabs, lens)[0] == oracle.ERR_ARG
    assert oracle.merge_kv_inplace(cfg, k, 3, 0, local, [None, insts[1]["pools"][0], None],
                                   tabs + [tabs[0]], lens + [lens[0]])[0] == oracle.ERR_ARG


def _remote_slots(tables, lens, g, m, P, B):
    """Slots of worker g's reshaped pool that receive remote heads, straight from the inputs:
    the distinct (block id, instance) pairs over the remote instances' in-range table cells."""
    slots = set()
    for g2 in range(m):
        if g2 == g:
            continue
        nb = (np.asarray(lens[g2], dtype=np.int64) + B - 1) // B
        for i, n in enumerate(nb):
            for b in tables[g2][i, :n]:
                if 0 <= b < P:
                    slots.add((int(b), g2))
    return slots


def test_remote_block_count_is_the_number_of_slots_filled():
    """The count reported next to the merge is the number of distinct slots of the reshaped
    pool that receive remote heads (Sec. 3.1, in-place migration: one slot per old block and
    instance): an id outside the pool has no slot, and a block two sequences of one instance
    share (a common prefix) is one slot.  Expected values come from the input tables alone,
    and from the bytes that actually changed in the pool."""
    m, k = 3, 1
    lens = [[13, 8, 9], [5, 22, 6], [16, 2, 7]]
    cfg, insts = make_instances(m, k, lens, n_heads=6, seed=11)
    P, B, S = cfg.src_pool_blocks, cfg.block_tokens, cfg.num_seqs
    tabs = [i["table"].copy() for i in insts]
    lns = [i["lens"] for i in insts]
    # instance 1: sequences 0 and 2 share their first block; instance 2: one id out of range
    tabs[1][2, 0] = tabs[1][0, 0]
    tabs[2][0, 1] = P + 3
    sub = cfg.n_kv_heads // m * 2 * B * cfg.head_dim
    for g in range(m):
        local = insts[g]["pools"][0].copy()
        remote = [None if g2 == g else insts[g2]["pools"][0] for g2 in range(m)]
        st, table, n = oracle.merge_kv_inplace(cfg, k, m, g, local, remote, tabs, lns)
        slots = _remote_slots(tabs, lns, g, m, P, B)
        assert st == oracle.ERR_BLOCK_ID
        assert n == len(slots)
        # fewer than the table cells of the remote instances: the shared block and, for the
        # workers that see instance 2 as remote, the bad id
        cells = sum(int(((np.asarray(lns[g2], dtype=np.int64) + B - 1) // B).sum())
                    for g2 in range(m) if g2 != g)
        assert n == cells - (1 if g != 1 else 0) - (1 if g != 2 else 0)
        # the bytes that changed lie inside exactly those slots (random payloads: a filled
        # slot differs from what was there)
        before = insts[g]["pools"][0].reshape(cfg.kv_layers, P * m, sub)
        after = local.reshape(cfg.kv_layers, P * m, sub)
        changed = {int(x) for x in np.nonzero((before != after).any(axis=(0, 2)))[0]}
        assert changed == {b * m + g2 for b, g2 in slots}
        # the shared block appears twice in the table with one id; the bad cell reads -1
        assert table[1 * S + 2, 0] == table[1 * S + 0, 0] == tabs[1][0, 0] * m + 1
        assert table[2 * S + 0, 1] == -1


def test_remote_block_count_on_a_clean_table_is_the_remote_cell_count():
    m, k = 4, 2
    lens = [[13, 1, 8, 0], [5, 22, 3, 9], [16, 2, 7, 7], [1, 1, 30, 4]]
    cfg, insts = make_instances(m, k, lens, n_heads=16, seed=4)
    B = cfg.block_tokens
    res = merge_all_ranks(cfg, insts, m, k)
    for r, (_, _, n) in res.items():
        g = r % m
        assert n == sum(int(((insts[g2]["lens"].astype(np.int64) + B - 1) // B).sum())
                        for g2 in range(m) if g2 != g)
