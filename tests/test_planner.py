"""Host logic of the library, no GPU needed: the C ABI loads and exports what the
header declares, the planner's segment table (interpreted here with numpy)
reproduces the oracle's shard byte for byte, and bad shapes are rejected."""
import itertools
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def shape_of(m: oracle.Model, **kw) -> ab.ModelShape:
    return ab.ModelShape(n_layers=m.n_layers, hidden=m.hidden, n_q_heads=m.n_q_heads,
                         n_kv_heads=m.n_kv_heads, head_dim=m.head_dim, ffn_dim=m.ffn_dim,
                         elem_bytes=m.elem_bytes, **kw)


def test_library_exports_every_declared_symbol():
    L = ab.lib()
    for header, exports in (("amoeba.h", ab.EXPORTS), ("amoeba_measure.h", ab.MEASURE_EXPORTS)):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        declared = set(re.findall(r"\b(amoeba_[a-z_]+)\s*\(", text))
        assert declared == set(exports), header
        for name in declared:
            assert hasattr(L, name), name
    # the product header stands alone: it neither includes nor mentions the measurement one
    product = open(os.path.join(ROOT, "include", "amoeba.h")).read()
    assert "amoeba_measure" not in product and "amoeba_plan_tune" not in product


def apply_segments(plan, src_shards, n_layers):
    """Interpret the plan's per-layer segment table on host byte arrays."""
    src_layer = ab.amoeba_plan_shard_bytes(plan, 0) // n_layers
    dst_layer = ab.amoeba_plan_shard_bytes(plan, 1) // n_layers
    dst = np.zeros(dst_layer * n_layers, dtype=np.uint8)
    hits = np.zeros(dst_layer * n_layers, dtype=np.uint8)
    for idx in range(ab.amoeba_plan_num_segments(plan)):
        r, so, sp, do, dp, rows, run = ab.amoeba_plan_segment(plan, idx)
        src = src_shards[r].view(np.uint8)
        for l in range(n_layers):
            for row in range(rows):
                a = l * src_layer + so + row * sp
                b = l * dst_layer + do + row * dp
                dst[b:b + run] = src[a:a + run]
                hits[b:b + run] += 1
    return dst, hits


PAIRS = list(itertools.product([1, 2, 4, 8], repeat=2)) + [(2, 3), (3, 2), (6, 4), (12, 8)]


@pytest.mark.parametrize("k,kp", PAIRS)
@pytest.mark.parametrize("n_kv", [24, 12])
def test_segment_table_reproduces_the_oracle(k, kp, n_kv):
    m = oracle.Model(n_layers=2, hidden=48, n_q_heads=24, n_kv_heads=n_kv, head_dim=4, ffn_dim=96,
                     elem_bytes=2)
    if n_kv % k or n_kv % kp:
        with pytest.raises(ab.AmoebaError):
            ab.amoeba_plan(shape_of(m), k, kp, 0)
        return
    n_src = oracle.shard_elems(m, k)
    src = [wl.random_bits(n_src, seed=100 + s) for s in range(k)]
    for rp in range(kp):
        plan = ab.amoeba_plan(shape_of(m), k, kp, rp)
        assert ab.amoeba_plan_shard_bytes(plan, 0) == n_src * 2
        assert ab.amoeba_plan_shard_bytes(plan, 1) == oracle.shard_elems(m, kp) * 2
        got, hits = apply_segments(plan, src, m.n_layers)
        assert (hits == 1).all()                 # every target byte has exactly one writer
        st, want = oracle.reshard_weights(m, k, kp, rp, src)
        assert st == oracle.OK
        np.testing.assert_array_equal(got.view(np.uint16), want)
        # the mask names exactly the ranks some segment reads
        mask = ab.amoeba_plan_src_rank_mask(plan)
        used = {ab.amoeba_plan_segment(plan, i)[0] for i in range(ab.amoeba_plan_num_segments(plan))}
        assert used == {r for r in range(k) if mask >> r & 1}
        # and the oracle agrees that the other ranks are not needed
        st, again = oracle.reshard_weights(
            m, k, kp, rp, [src[r] if r in used else None for r in range(k)])
        assert st == oracle.OK and (again == want).all()


def test_source_ranks_read_at_the_benchmark_configs():
    want = {"tiny": {0}, "llama7b": {2, 3}, "llama13b": {0, 1}, "gqa70b": {4, 5}, "long8b": {0}}
    for name in wl.ORDER:
        w = wl.WORKLOADS[name]
        s = ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
        plan = ab.amoeba_plan(s, w.src_tp, w.dst_tp, w.dst_rank)
        mask = ab.amoeba_plan_src_rank_mask(plan)
        assert {r for r in range(w.src_tp) if mask >> r & 1} == want[name]
        assert ab.amoeba_plan_kv_rank_mask(plan) == mask


def test_shard_bytes_at_7b_shape():
    w = wl.WORKLOADS["llama7b"]
    s = ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
    plan = ab.amoeba_plan(s, 4, 2, 1)
    per_layer = (4 * 4096 * 4096 + 3 * 4096 * 11008) * 2
    assert ab.amoeba_plan_shard_bytes(plan, 0) == 32 * per_layer // 4
    assert ab.amoeba_plan_shard_bytes(plan, 1) == 32 * per_layer // 2
    assert ab.amoeba_plan_kv_block_bytes(plan, 0) == 8 * 2 * 16 * 128 * 2
    assert ab.amoeba_plan_kv_block_bytes(plan, 1) == 16 * 2 * 16 * 128 * 2


def test_tensor_info_matches_the_packing_order():
    m = oracle.Model(2, 48, 24, 12, 4, 96, 2)
    plan = ab.amoeba_plan(shape_of(m), 2, 4, 1)
    for side, tp in ((0, 2), (1, 4)):
        at = 0
        shapes = [(24 * 4 // tp, 48), (12 * 4 // tp, 48), (12 * 4 // tp, 48), (48, 24 * 4 // tp),
                  (96 // tp, 48), (96 // tp, 48), (48, 96 // tp)]
        for t, (r, c) in enumerate(shapes):
            off, rows, cols, layer = ab.amoeba_plan_tensor_info(plan, side, t)
            assert (off, rows, cols) == (at, r, c)
            at += r * c
        assert layer == at == oracle.shard_elems(m, tp) // 2


@pytest.mark.parametrize("layout", [ab.KV_HEAD_MAJOR, ab.KV_TOKEN_MAJOR])
def test_kv_stride_order_matches_numpy_strides(layout):
    m = oracle.Model(1, 64, 8, 8, 16, 128, 2)
    s = shape_of(m, kv_block_tokens=4, kv_layout_src=layout, kv_layout_dst=layout)
    plan = ab.amoeba_plan(s, 2, 4, 0)
    for side, heads in ((0, 4), (1, 2)):
        sh, sc, st, sd, block = ab.amoeba_plan_kv_stride_order(plan, side)
        shape = (heads, 2, 4, 16) if layout == ab.KV_HEAD_MAJOR else (2, 4, heads, 16)
        a = np.zeros(shape, dtype=np.uint16)
        strides = [x // 2 for x in a.strides]
        if layout == ab.KV_HEAD_MAJOR:
            assert (sh, sc, st, sd) == tuple(strides)
        else:
            assert (sc, st, sh, sd) == tuple(strides)
        assert block == a.size


def test_plan_rejects_unsupported_shapes():
    good = dict(n_layers=2, hidden=48, n_q_heads=24, n_kv_heads=12, head_dim=4, ffn_dim=96)

    def bad(src_tp=1, dst_tp=2, rank=0, **kw):
        with pytest.raises(ab.AmoebaError):
            ab.amoeba_plan(ab.ModelShape(**{**good, **kw}), src_tp, dst_tp, rank)
        assert ab.amoeba_last_error() != ""

    bad(dst_tp=8)                      # 8 does not divide 12 kv heads
    bad(src_tp=5)
    bad(dst_tp=32, n_q_heads=64, n_kv_heads=64, ffn_dim=128)   # above the TP limit
    bad(rank=2)
    bad(rank=-1)
    bad(src_tp=0)
    bad(n_kv_heads=5)                  # q heads not a multiple of kv heads
    bad(elem_bytes=3)
    bad(kv_layout_dst=7)
    bad(n_layers=0)
    bad(dst_pool_blocks=2 ** 31)
    bad(ffn_dim=97)
    ab.amoeba_plan(ab.ModelShape(**good), 2, 3, 2)   # non-multiples are fine


def test_reshard_calls_reject_null_arguments_without_a_gpu():
    m = oracle.Model(1, 48, 24, 12, 4, 96, 2)
    plan = ab.amoeba_plan(shape_of(m), 1, 2, 0)
    assert ab.amoeba_reshard_weights(plan, [None], 4096, check=False) == ab.ERR_INVALID_ARG
    assert "NULL" in ab.amoeba_last_error()
    L = ab.lib()
    assert L.amoeba_reshard_weights(None, None, None, None) == ab.ERR_INVALID_ARG
    assert L.amoeba_reshard_kv(None, None, None, None, None, None, None) == ab.ERR_INVALID_ARG
    assert L.amoeba_plan_num_segments(None) == 0
    L.amoeba_plan_destroy(None)


def test_tune_rejects_unknown_knobs_and_bad_values():
    plan = ab.amoeba_plan(ab.ModelShape(2, 24, 8, 4, 4, 72), 1, 2, 0)
    for knob in range(10):
        ab.amoeba_plan_tune(plan, knob, 0)           # 0 restores the built-in choice
    for knob, value in [(10, 1), (-1, 1), (ab.TUNE_KV_SMALL_TABLE, 2), (ab.TUNE_KV_GRID, -5)]:
        with pytest.raises(ab.AmoebaError):
            ab.amoeba_plan_tune(plan, knob, value)
    assert "amoeba_plan_tune" in ab.amoeba_last_error()
    L = ab.lib()
    buf = (ctypes.c_void_p * 1)()
    assert L.amoeba_reshard_weights_part(plan.handle, buf, 8, 3, None) == ab.ERR_INVALID_ARG
    assert "AMOEBA_PART" in ab.amoeba_last_error()
    with pytest.raises(ab.AmoebaError):
        ab.amoeba_plan(ab.ModelShape(2, 24, 8, 4, 4, 72, kv_blocks_bound=-1), 1, 2, 0)


def test_workload_recipes_are_seeded_and_well_formed():
    for name in wl.ORDER:
        w = wl.WORKLOADS[name]
        lens = wl.seq_lens(w)
        assert (lens == wl.seq_lens(w)).all() and len(lens) == w.num_seqs and lens.min() >= 1
        table, pool = wl.block_placement(w, lens)
        nb = wl.blocks_per_seq(lens, w.block_tokens)
        used = table[table >= 0]
        assert len(used) == nb.sum() == len(set(used.tolist())) and used.max() < pool
        assert table.shape[1] % 8 == 0 and table.shape[1] >= nb.max()
        for i in range(len(lens)):
            assert (table[i, :nb[i]] >= 0).all() and (table[i, nb[i]:] == -1).all()
    assert wl.seq_lens(wl.WORKLOADS["long8b"])[:8].tolist() == [32768] * 8
    assert wl.seq_lens(wl.WORKLOADS["llama7b"]).max() <= 8192
