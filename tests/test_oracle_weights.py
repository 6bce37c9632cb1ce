"""Pins for the oracle's weight reshard (CPU only).

The oracle computes ranks and offsets with floor/mod arithmetic.  These tests
state the same problem through other means: np.split on the unsharded tensors,
torch.cat / torch.chunk, uniqueness of tags, round trips, and the FFN identity
of Sec. 3.2 Eq. (1)/(2).
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from helpers import full_model, reassemble, shard_of, unpack_shard

TPS_POW2 = [1, 2, 4, 8]
PAIRS = list(itertools.product(TPS_POW2, TPS_POW2)) + [(2, 3), (3, 2), (6, 4), (4, 6), (3, 12)]


def tiny_model(elem_bytes=2, n_kv=24, n_layers=2):
    return oracle.Model(n_layers=n_layers, hidden=48, n_q_heads=24, n_kv_heads=n_kv, head_dim=4,
                        ffn_dim=96, elem_bytes=elem_bytes)


def all_shards(layers, tp):
    return [shard_of(layers, tp, r) for r in range(tp)]


@pytest.mark.parametrize("k,kp", PAIRS)
def test_every_target_rank_equals_numpy_split_unique_tags(k, kp):
    """Brute force: every element of the model has its own 32-bit tag, so a wrong
    source rank, row, column, sub-block or layer shows up as a wrong tag."""
    m = tiny_model(elem_bytes=4)
    layers = full_model(m, unique=True)
    src = all_shards(layers, k)
    assert src[0].size == oracle.shard_elems(m, k)
    for rp in range(kp):
        st, dst = oracle.reshard_weights(m, k, kp, rp, src)
        assert st == oracle.OK
        np.testing.assert_array_equal(dst, shard_of(layers, kp, rp))


@pytest.mark.parametrize("n_kv", [24, 12, 6])
@pytest.mark.parametrize("k,kp", [(1, 2), (2, 1), (4, 2), (2, 6), (6, 3), (3, 1)])
def test_gqa_shapes_16bit(k, kp, n_kv):
    m = tiny_model(elem_bytes=2, n_kv=n_kv)
    layers = full_model(m, seed=k * 10 + kp)
    if n_kv % k or n_kv % kp:      # fewer kv heads than ranks (replication) is unsupported
        assert oracle.shard_elems(m, k if n_kv % k else kp) == -1
        return
    src = all_shards(layers, k)
    dsts = []
    for rp in range(kp):
        st, dst = oracle.reshard_weights(m, k, kp, rp, src)
        assert st == oracle.OK
        dsts.append(dst)
    # tiling: the k' target shards, un-fused and concatenated, are the unsharded model
    back = reassemble(dsts, m, kp)
    for l in range(m.n_layers):
        for name in layers[l]:
            np.testing.assert_array_equal(back[l][name], layers[l][name])


@pytest.mark.parametrize("k,kp", [(1, 4), (4, 2), (2, 3), (8, 1), (6, 4)])
def test_split_then_merge_round_trip(k, kp):
    m = tiny_model(elem_bytes=2)
    src = [oracle_random(m, k, seed=s) for s in range(k)]   # arbitrary shard bytes
    mid = [oracle.reshard_weights(m, k, kp, rp, src)[1] for rp in range(kp)]
    for r in range(k):
        st, back = oracle.reshard_weights(m, kp, k, r, mid)
        assert st == oracle.OK
        np.testing.assert_array_equal(back, src[r])


def oracle_random(m, tp, seed):
    n = oracle.shard_elems(m, tp)
    return np.random.default_rng(seed).integers(0, 65535, size=n, dtype=np.uint16, endpoint=True)


@pytest.mark.parametrize("elem_bytes", [1, 2, 4])
def test_special_cases_reduce_to_torch_routines(elem_bytes):
    """merge k->1 = torch.cat, split 1->k' = torch.chunk, k = k' = copy."""
    m = tiny_model(elem_bytes=elem_bytes)
    layers = full_model(m, seed=5)
    sview = {1: np.uint8, 2: np.int16, 4: np.int32}[elem_bytes]

    def T(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(sview))

    k = 4
    src = all_shards(layers, k)
    # merge 4 -> 1
    st, merged = oracle.reshard_weights(m, k, 1, 0, src)
    assert st == oracle.OK
    un_src = [unpack_shard(s, m, k) for s in src]
    un_dst = unpack_shard(merged, m, 1)
    for l in range(m.n_layers):
        for name in ("q", "k", "v", "g", "u"):
            ref = torch.cat([T(un_src[r][l][name]) for r in range(k)], dim=0)
            assert torch.equal(T(un_dst[l][name]), ref)
        for name in ("o", "d"):
            ref = torch.cat([T(un_src[r][l][name]) for r in range(k)], dim=1)
            assert torch.equal(T(un_dst[l][name]), ref)
    # split 1 -> 4
    one = all_shards(layers, 1)
    for rp in range(k):
        st, part = oracle.reshard_weights(m, 1, k, rp, one)
        un = unpack_shard(part, m, k)
        for l in range(m.n_layers):
            for name in ("q", "k", "v", "g", "u"):
                assert torch.equal(T(un[l][name]), torch.chunk(T(layers[l][name]), k, dim=0)[rp])
            for name in ("o", "d"):
                assert torch.equal(T(un[l][name]), torch.chunk(T(layers[l][name]), k, dim=1)[rp])
    # identity
    for r in range(k):
        st, same = oracle.reshard_weights(m, k, k, r, src)
        assert st == oracle.OK
        np.testing.assert_array_equal(same, src[r])


def test_ffn_and_attention_output_identity():
    """Sec. 3.2 Eq. (1)/(2): sum over ranks of f(x U_r) D_r equals f(x U) D, and the
    row-parallel o_proj sums the same way, on shards produced by the oracle."""
    m = oracle.Model(n_layers=1, hidden=16, n_q_heads=8, n_kv_heads=4, head_dim=4, ffn_dim=24,
                     elem_bytes=4)
    rng = np.random.default_rng(3)
    layers = full_model(m, seed=0)
    for name in layers[0]:       # replace opaque bits by real float32 weights
        w = rng.standard_normal(layers[0][name].shape).astype(np.float32)
        layers[0][name] = w.view(np.uint32)
    f = lambda a: a / (1.0 + np.exp(-a))      # SiLU
    x = rng.standard_normal((5, m.hidden))
    W = {n: layers[0][n].view(np.float32).astype(np.float64) for n in layers[0]}
    ffn_full = (f(x @ W["g"].T) * (x @ W["u"].T)) @ W["d"].T
    a = rng.standard_normal((5, m.n_q_heads * m.head_dim))
    attn_full = a @ W["o"].T
    for k, kp in [(1, 4), (4, 2), (2, 1), (2, 4)]:
        src = all_shards(layers, k)
        ffn_sum, attn_sum = 0.0, 0.0
        for rp in range(kp):
            st, dst = oracle.reshard_weights(m, k, kp, rp, src)
            assert st == oracle.OK
            t = unpack_shard(dst, m, kp)[0]
            g, u, d_, o = (t[n].view(np.float32).astype(np.float64) for n in ("g", "u", "d", "o"))
            ffn_sum = ffn_sum + (f(x @ g.T) * (x @ u.T)) @ d_.T
            cols = m.n_q_heads * m.head_dim // kp
            attn_sum = attn_sum + a[:, rp * cols:(rp + 1) * cols] @ o.T
        np.testing.assert_allclose(ffn_sum, ffn_full, rtol=1e-9, atol=1e-9)
        np.testing.assert_allclose(attn_sum, attn_full, rtol=1e-9, atol=1e-9)


def test_q_head_rows_follow_the_head_range_rule():
    """Sec. 3.1 rule applied to q heads: 1-based worker i owns heads
    (H/TP)(i-1)+1 .. (H/TP)(i-1)+H/TP.  Each q row is tagged with its 1-based head."""
    m = oracle.Model(n_layers=1, hidden=4, n_q_heads=8, n_kv_heads=8, head_dim=2, ffn_dim=8,
                     elem_bytes=2)
    layers = full_model(m, seed=1)
    head_of_row = np.repeat(np.arange(1, 9, dtype=np.uint16), m.head_dim)
    layers[0]["q"][:] = head_of_row[:, None]
    src = all_shards(layers, 1)
    TP = 4
    for i in range(1, TP + 1):
        st, dst = oracle.reshard_weights(m, 1, TP, i - 1, src)
        q = unpack_shard(dst, m, TP)[0]["q"]
        lo, hi = (8 // TP) * (i - 1) + 1, (8 // TP) * (i - 1) + 8 // TP
        assert sorted(set(q.ravel().tolist())) == list(range(lo, hi + 1))


def test_unneeded_source_ranks_may_be_null_and_needed_may_not():
    m = tiny_model()
    layers = full_model(m, seed=2)
    src = all_shards(layers, 4)
    # target rank 1 of TP2 is built from source ranks 2 and 3 of TP4 only
    st, dst = oracle.reshard_weights(m, 4, 2, 1, [None, None, src[2], src[3]])
    assert st == oracle.OK
    np.testing.assert_array_equal(dst, shard_of(layers, 2, 1))
    st, _ = oracle.reshard_weights(m, 4, 2, 1, [src[0], src[1], None, src[3]])
    assert st == oracle.ERR_ARG


def test_rejects_bad_arguments():
    m = tiny_model(n_kv=12)
    assert oracle.shard_elems(m, 8) == -1          # 8 does not divide 12 kv heads
    src = [np.zeros(oracle.shard_elems(m, 1), np.uint16)]
    assert oracle.reshard_weights(m, 1, 8, 0, src)[0] == oracle.ERR_ARG
    assert oracle.reshard_weights(m, 1, 2, 2, src)[0] == oracle.ERR_ARG
    assert oracle.reshard_weights(m, 1, 2, -1, src)[0] == oracle.ERR_ARG
    assert oracle.reshard_weights(m, 0, 2, 0, src)[0] == oracle.ERR_ARG
    bad = oracle.Model(2, 48, 24, 5, 4, 96, 2)     # q heads not a multiple of kv heads
    assert oracle.shard_elems(bad, 1) == -1


def test_shard_sizes_closed_form():
    """Even distribution (Sec. 2.2): a rank holds 1/tp of every sharded tensor."""
    m = oracle.Model(n_layers=32, hidden=4096, n_q_heads=32, n_kv_heads=32, head_dim=128,
                     ffn_dim=11008, elem_bytes=2)
    per_layer = 4 * 4096 * 4096 + 3 * 4096 * 11008
    for tp in (1, 2, 4, 8):
        assert oracle.shard_elems(m, tp) == 32 * per_layer // tp


def test_writes_exactly_the_destination_shard():
    m = tiny_model()
    layers = full_model(m, seed=7)
    src = all_shards(layers, 2)
    n = oracle.shard_elems(m, 4)
    buf = np.full(n + 64, 0xDEAD, dtype=np.uint16)
    st, _ = oracle.reshard_weights(m, 2, 4, 3, src, dst=buf[32:32 + n])
    assert st == oracle.OK
    assert (buf[:32] == 0xDEAD).all() and (buf[32 + n:] == 0xDEAD).all()
    np.testing.assert_array_equal(buf[32:32 + n], shard_of(layers, 4, 3))
