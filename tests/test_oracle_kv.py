"""Pins for the oracle's KV regroup and table rewrite (CPU only).

The oracle indexes blocks with closed-form offsets.  Here the same cache is
paged out and read back with numpy reshape/transpose (helpers.page_out /
page_in), so the pins are independent of the oracle's index formulas.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from helpers import HEAD_MAJOR, TOKEN_MAJOR, logical_kv, page_in, page_out, random_table

LAYOUTS = [HEAD_MAJOR, TOKEN_MAJOR]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_all_ranks(kv_cfg, k, kp, src_pools, table, lens, sentinel=0xABCD):
    """Reshard for every target rank; returns (pools, tables, totals)."""
    be = oracle.kv_block_elems(kv_cfg, kp)
    pools, tables, totals = [], [], []
    for rp in range(kp):
        dst = np.full((kv_cfg.kv_layers, kv_cfg.dst_pool_blocks, be), sentinel, dtype=np.uint16)
        st, dt, total = oracle.reshard_kv(kv_cfg, k, kp, rp, src_pools, table, lens, dst)
        assert st == oracle.OK
        pools.append(dst), tables.append(dt), totals.append(total)
    return pools, tables, totals


def make_case(k, lay_s, lay_d, lens, n_heads=8, d=4, B=4, layers=2, seed=0, slack=3):
    lens = np.asarray(lens, dtype=np.int32)
    nb = (lens.astype(np.int64) + B - 1) // B
    src_pool_blocks = int(nb.sum()) + 5
    table = random_table(lens, B, src_pool_blocks, seed=seed)
    kv = logical_kv(layers, lens, n_heads, d, np.uint16, seed=seed)
    src_pools = page_out(kv, lens, table, src_pool_blocks, k, lay_s, B)
    cfg = oracle.KV(kv_layers=layers, n_kv_heads=n_heads, head_dim=d, block_tokens=B,
                    num_seqs=len(lens), max_blocks_per_seq=table.shape[1],
                    src_pool_blocks=src_pool_blocks, dst_pool_blocks=int(nb.sum()) + slack,
                    layout_src=lay_s, layout_dst=lay_d)
    return cfg, kv, src_pools, table, lens, nb


def test_worked_example_of_the_paper_h8_tp4():
    """Sec. 3.1: H = 8, TP4 -> W2 keeps H3,H4; (H1,H2)/(H5,H6)/(H7,H8) go to W1/W3/W4.
    Every K/V element is tagged with its 1-based head number; after the oracle's
    TP1 -> TP4 reshard, worker Wi's pool must hold exactly the heads the text lists."""
    want = {}
    for line in open(os.path.join(GOLDEN, "kv_head_ranges_H8_TP4.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w, heads = line.split(":")
        want[int(w.strip()[1:])] = sorted(int(h[1:]) for h in heads.split())
    assert want[2] == [3, 4]
    B, d, H = 4, 2, 8
    lens = np.array([9, 4, 1], dtype=np.int32)
    for lay_s, lay_d in itertools.product(LAYOUTS, LAYOUTS):
        cfg, kv, _, table, lens, nb = make_case(1, lay_s, lay_d, lens, n_heads=H, d=d, B=B)
        for l in range(len(kv)):
            for a in kv[l]:
                a[:] = np.arange(1, H + 1, dtype=np.uint16)[None, :, None, None]
        src_pools = page_out(kv, lens, table, cfg.src_pool_blocks, 1, lay_s, B)
        for worker in range(1, 5):
            be = oracle.kv_block_elems(cfg, 4)
            dst = np.zeros((cfg.kv_layers, cfg.dst_pool_blocks, be), dtype=np.uint16)
            st, dt, total = oracle.reshard_kv(cfg, 1, 4, worker - 1, src_pools, table, lens, dst)
            assert st == oracle.OK
            # look only at real tokens: read the worker's pool as a TP1 cache of 2 heads
            got = page_in([dst], lens, dt, 1, lay_d, B, 2, d)
            seen = sorted(set(np.concatenate([a.ravel() for row in got for a in row]).tolist()))
            assert seen == want[worker]


@pytest.mark.parametrize("k,kp", [(1, 4), (4, 1), (4, 2), (2, 4), (8, 4), (2, 2), (1, 1)])
@pytest.mark.parametrize("lay_s,lay_d", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_every_token_head_value_is_preserved(k, kp, lay_s, lay_d):
    """Assignment-agnostic: reading (dst table, dst pools of all k' ranks) gives back the
    logical cache the source pools were built from."""
    cfg, kv, src_pools, table, lens, nb = make_case(k, lay_s, lay_d, [13, 1, 8, 0, 22, 5],
                                                    seed=k * 7 + kp)
    pools, tables, totals = run_all_ranks(cfg, k, kp, src_pools, table, lens)
    for t in tables[1:]:
        np.testing.assert_array_equal(t, tables[0])      # the scan does not depend on the rank
    back = page_in(pools, lens, tables[0], kp, lay_d, cfg.block_tokens, cfg.n_kv_heads,
                   cfg.head_dim)
    for l in range(cfg.kv_layers):
        for i in range(len(lens)):
            np.testing.assert_array_equal(back[l][i], kv[l][i])
    assert totals == [int(nb.sum())] * kp


@pytest.mark.parametrize("k,kp", [(2, 3), (3, 2), (6, 4), (3, 12)])
def test_tp_degrees_that_do_not_divide_each_other(k, kp):
    cfg, kv, src_pools, table, lens, nb = make_case(k, HEAD_MAJOR, HEAD_MAJOR, [7, 12, 3],
                                                    n_heads=12, seed=kp)
    pools, tables, _ = run_all_ranks(cfg, k, kp, src_pools, table, lens)
    back = page_in(pools, lens, tables[0], kp, HEAD_MAJOR, cfg.block_tokens, 12, cfg.head_dim)
    for l in range(cfg.kv_layers):
        for i in range(len(lens)):
            np.testing.assert_array_equal(back[l][i], kv[l][i])


def test_table_is_the_exclusive_scan_and_unused_blocks_are_untouched():
    lens = [13, 1, 8, 0, 22, 5]
    cfg, kv, src_pools, table, lens, nb = make_case(2, HEAD_MAJOR, HEAD_MAJOR, lens, slack=4)
    pools, tables, totals = run_all_ranks(cfg, 2, 4, src_pools, table, lens, sentinel=0x5A5A)
    t = tables[0]
    W = t.shape[1]
    base = np.concatenate([[0], np.cumsum(nb)[:-1]])
    for i in range(len(lens)):
        np.testing.assert_array_equal(t[i, :nb[i]], base[i] + np.arange(nb[i]))
        assert (t[i, nb[i]:] == -1).all()
    used = t[t >= 0]
    assert sorted(used.tolist()) == list(range(int(nb.sum())))   # bijection onto [0, total)
    assert (t[3] == -1).all() and W >= nb.max()                  # empty sequence -> empty row
    for p in pools:
        assert (p[:, int(nb.sum()):] == 0x5A5A).all()            # pool blocks past the total


def test_whole_blocks_move_including_slots_past_the_sequence_end():
    """Slots after the last token are copied verbatim (the source filler comes along)."""
    cfg, kv, src_pools, table, lens, nb = make_case(1, HEAD_MAJOR, HEAD_MAJOR, [5], n_heads=2,
                                                    layers=1)
    pools, tables, _ = run_all_ranks(cfg, 1, 1, src_pools, table, lens)
    for j in range(int(nb[0])):
        np.testing.assert_array_equal(pools[0][0, tables[0][0, j]], src_pools[0][0, table[0, j]])


@pytest.mark.parametrize("layout", LAYOUTS)
def test_same_tp_same_layout_is_index_select_by_table(layout):
    cfg, kv, src_pools, table, lens, nb = make_case(2, layout, layout, [9, 16, 2], seed=4)
    pools, tables, _ = run_all_ranks(cfg, 2, 2, src_pools, table, lens)
    order = np.concatenate([table[i, :nb[i]] for i in range(len(lens))]).astype(np.int64)
    for r in range(2):
        for l in range(cfg.kv_layers):
            ref = torch.index_select(torch.from_numpy(src_pools[r][l].view(np.int16)), 0,
                                     torch.from_numpy(order))
            got = torch.from_numpy(pools[r][l, :len(order)].view(np.int16))
            assert torch.equal(got, ref)


def test_round_trip_k_kp_k_and_second_compaction_is_identity():
    cfg, kv, src_pools, table, lens, nb = make_case(2, HEAD_MAJOR, TOKEN_MAJOR, [13, 1, 8, 22],
                                                    seed=11)
    mid_pools, mid_tables, _ = run_all_ranks(cfg, 2, 4, src_pools, table, lens)
    total = int(nb.sum())
    back_cfg = oracle.KV(kv_layers=cfg.kv_layers, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                         block_tokens=cfg.block_tokens, num_seqs=cfg.num_seqs,
                         max_blocks_per_seq=cfg.max_blocks_per_seq,
                         src_pool_blocks=cfg.dst_pool_blocks, dst_pool_blocks=total,
                         layout_src=TOKEN_MAJOR, layout_dst=HEAD_MAJOR)
    pools, tables, _ = run_all_ranks(back_cfg, 4, 2, mid_pools, mid_tables[0], lens)
    # back at TP2 / header-centric: block b of the compacted pool is source block table[i][j]
    order = np.concatenate([table[i, :nb[i]] for i in range(len(lens))])
    for r in range(2):
        np.testing.assert_array_equal(pools[r], src_pools[r][:, order])
    np.testing.assert_array_equal(tables[0], mid_tables[0])      # already compact: same ids
    # applying the same-TP compaction to a compact pool changes nothing
    again_cfg = oracle.KV(kv_layers=cfg.kv_layers, n_kv_heads=cfg.n_kv_heads,
                          head_dim=cfg.head_dim, block_tokens=cfg.block_tokens,
                          num_seqs=cfg.num_seqs, max_blocks_per_seq=cfg.max_blocks_per_seq,
                          src_pool_blocks=total, dst_pool_blocks=total)
    pools2, tables2, _ = run_all_ranks(again_cfg, 2, 2, pools, tables[0], lens)
    for r in range(2):
        np.testing.assert_array_equal(pools2[r], pools[r])
    np.testing.assert_array_equal(tables2[0], tables[0])


def test_head_range_closed_form_for_every_rank():
    """Sec. 3.1: 1-based worker i of TP owns heads (H/TP)(i-1)+1 .. (H/TP)(i-1)+H/TP."""
    H, B, d = 12, 2, 2
    lens = np.array([3], dtype=np.int32)
    for k, kp in itertools.product([1, 2, 3, 4, 6, 12], repeat=2):
        cfg, kv, _, table, lens, nb = make_case(k, HEAD_MAJOR, HEAD_MAJOR, lens, n_heads=H, d=d,
                                                B=B, layers=1)
        for a in kv[0]:
            a[:] = np.arange(1, H + 1, dtype=np.uint16)[None, :, None, None]
        src_pools = page_out(kv, lens, table, cfg.src_pool_blocks, k, HEAD_MAJOR, B)
        for i in range(1, kp + 1):
            dst = np.zeros((1, cfg.dst_pool_blocks, oracle.kv_block_elems(cfg, kp)), np.uint16)
            st, dt, _ = oracle.reshard_kv(cfg, k, kp, i - 1, src_pools, table, lens, dst)
            assert st == oracle.OK
            got = page_in([dst], lens, dt, 1, HEAD_MAJOR, B, H // kp, d)[0][0]
            lo, hi = (H // kp) * (i - 1) + 1, (H // kp) * (i - 1) + H // kp
            np.testing.assert_array_equal(got[0, :, 0, 0], np.arange(lo, hi + 1))


def test_overflow_conditions_write_nothing_and_clear_the_table():
    cfg, kv, src_pools, table, lens, nb = make_case(1, HEAD_MAJOR, HEAD_MAJOR, [13, 8])
    be = oracle.kv_block_elems(cfg, 2)
    total = int(nb.sum())

    def attempt(c, lens_):
        dst = np.full((c.kv_layers, max(c.dst_pool_blocks, 1), be), 0x7777, dtype=np.uint16)
        st, dt, tot = oracle.reshard_kv(c, 1, 2, 0, src_pools, table[:, :c.max_blocks_per_seq]
                                        if c.max_blocks_per_seq <= table.shape[1] else table,
                                        lens_, dst)
        return st, dt, tot, dst

    import dataclasses
    small_pool = dataclasses.replace(cfg, dst_pool_blocks=total - 1)
    st, dt, tot, dst = attempt(small_pool, lens)
    assert st == oracle.ERR_OVERFLOW and tot == 0 and (dt == -1).all() and (dst == 0x7777).all()
    narrow = dataclasses.replace(cfg, max_blocks_per_seq=int(nb.max()) - 1)
    st, dt, tot, dst = attempt(narrow, lens)
    assert st == oracle.ERR_OVERFLOW and (dt == -1).all() and (dst == 0x7777).all()
    neg = lens.copy()
    neg[1] = -3
    st, dt, tot, dst = attempt(cfg, neg)
    assert st == oracle.ERR_OVERFLOW and (dt == -1).all() and (dst == 0x7777).all()
    exact = dataclasses.replace(cfg, dst_pool_blocks=total)
    st, dt, tot, dst = attempt(exact, lens)
    assert st == oracle.OK and tot == total


def test_out_of_range_source_block_is_skipped_and_reported():
    cfg, kv, src_pools, table, lens, nb = make_case(1, HEAD_MAJOR, HEAD_MAJOR, [9, 6], layers=1)
    be = oracle.kv_block_elems(cfg, 1)
    good = np.full((1, cfg.dst_pool_blocks, be), 0x1111, dtype=np.uint16)
    oracle.reshard_kv(cfg, 1, 1, 0, src_pools, table, lens, good)
    bad_table = table.copy()
    bad_table[0, 1] = cfg.src_pool_blocks          # one id past the pool
    dst = np.full((1, cfg.dst_pool_blocks, be), 0x1111, dtype=np.uint16)
    st, dt, tot = oracle.reshard_kv(cfg, 1, 1, 0, src_pools, bad_table, lens, dst)
    assert st == oracle.ERR_BLOCK_ID
    assert (dst[0, 1] == 0x1111).all()             # the offending block was not written
    mask = np.ones(cfg.dst_pool_blocks, bool)
    mask[1] = False
    np.testing.assert_array_equal(dst[0, mask], good[0, mask])


def test_rejects_bad_arguments():
    cfg, kv, src_pools, table, lens, nb = make_case(1, HEAD_MAJOR, HEAD_MAJOR, [4], n_heads=6)
    dst = np.zeros((cfg.kv_layers, cfg.dst_pool_blocks, 1024), np.uint16)
    assert oracle.kv_block_elems(cfg, 4) == -1
    assert oracle.reshard_kv(cfg, 1, 4, 0, src_pools, table, lens, dst)[0] == oracle.ERR_ARG
    assert oracle.reshard_kv(cfg, 1, 2, 2, src_pools, table, lens, dst)[0] == oracle.ERR_ARG
    assert oracle.reshard_kv(cfg, 1, 2, 0, [None], table, lens, dst)[0] == oracle.ERR_ARG
    import dataclasses
    bad_layout = dataclasses.replace(cfg, layout_dst=2)
    assert oracle.reshard_kv(bad_layout, 1, 2, 0, src_pools, table, lens, dst)[0] == oracle.ERR_ARG


def test_only_owner_ranks_are_needed():
    cfg, kv, src_pools, table, lens, nb = make_case(4, HEAD_MAJOR, HEAD_MAJOR, [9, 3])
    be = oracle.kv_block_elems(cfg, 2)
    full = np.zeros((cfg.kv_layers, cfg.dst_pool_blocks, be), np.uint16)
    part = np.zeros_like(full)
    assert oracle.reshard_kv(cfg, 4, 2, 1, src_pools, table, lens, full)[0] == oracle.OK
    st, _, _ = oracle.reshard_kv(cfg, 4, 2, 1, [None, None, src_pools[2], src_pools[3]], table,
                                 lens, part)
    assert st == oracle.OK
    np.testing.assert_array_equal(full, part)


@pytest.mark.parametrize("elem_bytes", [1, 4])
def test_other_element_widths(elem_bytes):
    dt = {1: np.uint8, 4: np.uint32}[elem_bytes]
    lens = np.array([7, 2], dtype=np.int32)
    B, d, H = 4, 4, 4
    nb = (lens + B - 1) // B
    table = random_table(lens, B, 8, seed=1)
    kv = logical_kv(1, lens, H, d, dt, seed=2)
    src_pools = page_out(kv, lens, table, 8, 2, TOKEN_MAJOR, B)
    cfg = oracle.KV(kv_layers=1, n_kv_heads=H, head_dim=d, block_tokens=B, num_seqs=2,
                    max_blocks_per_seq=table.shape[1], src_pool_blocks=8,
                    dst_pool_blocks=int(nb.sum()), layout_src=TOKEN_MAJOR, layout_dst=HEAD_MAJOR,
                    elem_bytes=elem_bytes)
    dst = np.zeros((1, cfg.dst_pool_blocks, oracle.kv_block_elems(cfg, 1)), dt)
    st, t, _ = oracle.reshard_kv(cfg, 2, 1, 0, src_pools, table, lens, dst)
    assert st == oracle.OK
    back = page_in([dst], lens, t, 1, HEAD_MAJOR, B, H, d)
    for i in range(2):
        np.testing.assert_array_equal(back[0][i], kv[0][i])
