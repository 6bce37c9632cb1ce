"""Seeded random shapes through the host planner, no GPU: for every draw the segment table,
interpreted with numpy, must write every target byte exactly once and reproduce the oracle's
shard (dense, padded and expert-wise layouts; 1-, 2- and 4-byte elements; degree pairs that
are multiples, divisors and neither)."""
import numpy as np
import pytest

import oracle
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl
from test_planner_padded import apply_segments

DEGREES = [1, 2, 3, 4, 6, 8, 12, 16]


def draw(seed):
    rng = np.random.default_rng(1000 + seed)
    k, kp = (int(x) for x in rng.choice(DEGREES, size=2))
    lcm = int(np.lcm(k, kp))
    group = int(rng.integers(1, 4))                      # q heads per kv head
    n_kv = lcm * int(rng.integers(1, 3))
    eb = int(rng.choice([1, 2, 4]))
    m = oracle.Model(n_layers=int(rng.integers(1, 4)), hidden=int(rng.integers(1, 9)) * 4,
                     n_q_heads=n_kv * group, n_kv_heads=n_kv, head_dim=int(rng.integers(1, 6)),
                     ffn_dim=lcm * int(rng.integers(1, 5)), elem_bytes=eb)
    return rng, m, k, kp, int(rng.integers(0, kp))


def shape(m, **kw):
    return ab.ModelShape(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_dim,
                         elem_bytes=m.elem_bytes, **kw)


def compare(plan, src, want, m):
    assert ab.amoeba_plan_shard_bytes(plan, 1) == want.nbytes
    assert ab.amoeba_plan_shard_bytes(plan, 0) == src[0].nbytes
    got, hits = apply_segments(plan, src, m.n_layers)
    assert (hits == 1).all()
    np.testing.assert_array_equal(got, want.view(np.uint8))


@pytest.mark.parametrize("seed", range(40))
def test_dense_plans(seed):
    _, m, k, kp, rp = draw(seed)
    src = [wl.random_bits(oracle.shard_elems(m, k), seed=seed * 17 + r, elem_bytes=m.elem_bytes)
           for r in range(k)]
    st, want = oracle.reshard_weights(m, k, kp, rp, src)
    assert st == oracle.OK
    compare(ab.amoeba_plan(shape(m), k, kp, rp), src, want, m)


@pytest.mark.parametrize("seed", range(40))
def test_padded_plans(seed):
    rng, m, k, kp, rp = draw(seed)
    T = int(np.lcm(k, kp))
    if T > ab.MAX_TP:
        with pytest.raises(ab.AmoebaError):
            ab.amoeba_plan(shape(m, w_layout_dst=1, pad_max_tp=T, pad_page_bytes=64), k, kp, rp)
        return
    page = m.elem_bytes * int(rng.integers(1, 200))
    sp, dp = [(False, True), (True, True), (True, False)][seed % 3]
    dense = [wl.random_bits(oracle.shard_elems(m, k), seed=seed * 19 + r, elem_bytes=m.elem_bytes)
             for r in range(k)]
    src = dense
    if sp:
        up = oracle.Pad(T, page, src_padded=False, dst_padded=True)
        src = [oracle.reshard_weights_padded(m, up, k, k, r, dense)[1] for r in range(k)]
    st, want = oracle.reshard_weights_padded(m, oracle.Pad(T, page, sp, dp), k, kp, rp, src)
    assert st == oracle.OK
    plan = ab.amoeba_plan(shape(m, w_layout_src=int(sp), w_layout_dst=int(dp), pad_max_tp=T,
                                pad_page_bytes=page), k, kp, rp)
    compare(plan, src, want, m)


@pytest.mark.parametrize("seed", range(40))
def test_expert_plans(seed):
    rng, m, k, kp, rp = draw(seed)
    n_exp = int(np.lcm(k, kp)) * int(rng.integers(1, 4))
    page = m.elem_bytes * int(rng.integers(1, 200))
    sp, dp = [(False, False), (False, True), (True, True), (True, False)][seed % 4]
    flat = oracle.Moe(n_exp)
    dense = [wl.random_bits(oracle.moe_shard_elems(m, flat, False, k), seed=seed * 23 + r,
                            elem_bytes=m.elem_bytes) for r in range(k)]
    src = dense
    if sp:
        up = oracle.Moe(n_exp, page, False, True)
        src = [oracle.reshard_weights_moe(m, up, k, k, r, dense)[1] for r in range(k)]
    st, want = oracle.reshard_weights_moe(m, oracle.Moe(n_exp, page, sp, dp), k, kp, rp, src)
    assert st == oracle.OK
    plan = ab.amoeba_plan(shape(m, w_layout_src=int(sp), w_layout_dst=int(dp), n_experts=n_exp,
                                pad_page_bytes=page), k, kp, rp)
    compare(plan, src, want, m)
