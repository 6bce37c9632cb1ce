"""Pins for the oracle's mixture-of-experts reshard (Sec. 3.2, EP discussion; the
TPkEPk configurations of Sec. 4.3), CPU only.

The expert-wise shard is rebuilt here with np.split, list slicing, np.zeros and concatenation;
page counts are checked against the MoE rows of the paper's Table 2; a routed FFN computed from
the resharded ranks is compared with the one computed from the unsharded experts.
"""
import os

import numpy as np
import pytest

import oracle
from moe_helpers import moe_full_model, moe_shard_of

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

# degrees 1, 2, 3, 4, 6, 8 divide the heads and the 24 experts; none but 1 divides ffn_dim = 5
MODEL = oracle.Model(n_layers=2, hidden=12, n_q_heads=24, n_kv_heads=24, head_dim=2, ffn_dim=5,
                     elem_bytes=2)
E = 24


@pytest.mark.parametrize("page", [0, 64, 1000, 2])
@pytest.mark.parametrize("k,kp", [(1, 1), (1, 4), (4, 1), (2, 8), (8, 2), (2, 3), (3, 2), (6, 4),
                                  (4, 4)])
def test_every_layout_pair_matches_numpy_packing(page, k, kp):
    layers = moe_full_model(MODEL, E, seed=page + 10 * k + kp)
    pe = page // 2
    dense_src = [moe_shard_of(layers, k, r, E, 0) for r in range(k)]
    padded_src = [moe_shard_of(layers, k, r, E, pe) for r in range(k)]
    for rp in range(kp):
        for sp, dp in [(False, False), (False, True), (True, True), (True, False)]:
            if page == 0 and (sp or dp):
                continue
            x = oracle.Moe(E, page, sp, dp)
            st, got = oracle.reshard_weights_moe(MODEL, x, k, kp, rp, padded_src if sp else dense_src)
            assert st == oracle.OK
            want = moe_shard_of(layers, kp, rp, E, pe if dp else 0)
            assert got.size == want.size == oracle.moe_shard_elems(MODEL, x, dp, kp)
            np.testing.assert_array_equal(got, want)


def test_unique_tags_every_expert_lands_once():
    """With a distinct 32-bit tag on every element of the model, the target shards of all ranks
    together hold every tag exactly once (nothing dropped, nothing duplicated)."""
    m = oracle.Model(n_layers=1, hidden=8, n_q_heads=8, n_kv_heads=8, head_dim=2, ffn_dim=3,
                     elem_bytes=4)
    layers = moe_full_model(m, 8, unique=True)
    total = sum(a.size for a in [layers[0][n] for n in "qkvo"]) + \
        sum(t.size for ex in layers[0]["experts"] for t in ex)
    for k, kp in [(1, 8), (8, 1), (2, 4), (4, 2), (8, 8)]:
        src = [moe_shard_of(layers, k, r, 8, 0) for r in range(k)]
        seen = np.concatenate([oracle.reshard_weights_moe(m, oracle.Moe(8), k, kp, rp, src)[1]
                               for rp in range(kp)])
        assert seen.size == total
        np.testing.assert_array_equal(np.sort(seen), np.arange(total, dtype=np.uint32))


def test_round_trip_restores_every_source_shard():
    layers = moe_full_model(MODEL, E, seed=5)
    for k, kp, page in [(2, 8, 0), (3, 4, 64), (8, 1, 1000)]:
        pe = page // 2
        x = oracle.Moe(E, page, bool(page), bool(page))
        src = [moe_shard_of(layers, k, r, E, pe) for r in range(k)]
        mid = [oracle.reshard_weights_moe(MODEL, x, k, kp, rp, src)[1] for rp in range(kp)]
        for r in range(k):
            st, back = oracle.reshard_weights_moe(MODEL, x, kp, k, r, mid)
            assert st == oracle.OK
            np.testing.assert_array_equal(back, src[r])


def test_scale_up_is_a_contiguous_range_of_one_source_rank():
    """k | k': the target's experts are one byte range of the hosting source rank's layer, so
    the experts that leave are released and nothing is copied (Sec. 3.2: unused expert weights
    are freed directly).  With padding the range is page aligned."""
    layers = moe_full_model(MODEL, E, seed=3)
    for page in (0, 64):
        pe = page // 2
        x = oracle.Moe(E, page, bool(page), bool(page))
        for k, kp in [(1, 4), (2, 8), (1, 3), (4, 8)]:
            own_s, first_s, tensor, slot, layer_s = oracle.moe_geometry(MODEL, x, bool(page), k)
            own_d, first_d, _, _, layer_d = oracle.moe_geometry(MODEL, x, bool(page), kp)
            assert own_s == E // k and own_d == E // kp and tensor == MODEL.ffn_dim * MODEL.hidden
            src = [moe_shard_of(layers, k, r, E, pe) for r in range(k)]
            for rp in range(kp):
                host = rp * k // kp
                st, dst = oracle.reshard_weights_moe(MODEL, x, k, kp, rp, src)
                lo = first_s + (rp * own_d - host * own_s) * slot
                n = own_d * slot
                if page:
                    assert lo % pe == 0 and n % pe == 0 and first_d % pe == 0
                np.testing.assert_array_equal(
                    dst.reshape(MODEL.n_layers, layer_d)[:, first_d:],
                    src[host].reshape(MODEL.n_layers, layer_s)[:, lo:lo + n])


def test_expert_pages_reproduce_table_2():
    """MoE rows of Table 2: pages of one projection summed over the experts of a rank, at
    EP1 (all experts) and EP4 (a quarter of them), 2 MiB pages, 16-bit weights."""
    page = 2 * 1024 * 1024
    rows = 0
    for line in open(os.path.join(GOLDEN, "ffn_pages_table2.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, hidden, inter, experts, p1, p4 = line.split()
        if experts == "-":
            continue
        rows += 1
        m = oracle.Model(n_layers=1, hidden=int(hidden), n_q_heads=8, n_kv_heads=8, head_dim=8,
                         ffn_dim=int(inter), elem_bytes=2)
        x = oracle.Moe(int(experts), page, True, True)
        for tp, want in ((1, float(p1)), (4, float(p4))):
            own, first, tensor, slot, layer = oracle.moe_geometry(m, x, True, tp)
            assert own * tensor * 2 / page == pytest.approx(want, abs=1e-3), name
            # an expert of 3 x 7.91 pages occupies 24: below one page of waste per expert
            assert slot * 2 % page == 0 and 0 <= (slot - 3 * tensor) * 2 < page
            assert layer == first + own * slot and first * 2 % page == 0
    assert rows == 2


def test_routed_ffn_from_resharded_ranks_equals_the_unsharded_one():
    """Expert parallelism: every rank evaluates the experts it owns on the tokens routed to
    them and the partial outputs are summed over ranks.  Computed from the oracle's shards
    (any degree, with or without padding) this equals the routed FFN of the unsharded
    model."""
    m = oracle.Model(n_layers=1, hidden=8, n_q_heads=8, n_kv_heads=8, head_dim=2, ffn_dim=6,
                     elem_bytes=4)
    n_exp = 8
    rng = np.random.default_rng(1)
    layers = moe_full_model(m, n_exp, seed=0)
    L = layers[0]
    for n in "qkvo":
        L[n] = rng.standard_normal(L[n].shape).astype(np.float32).view(np.uint32)
    L["experts"] = [tuple(rng.standard_normal(t.shape).astype(np.float32).view(np.uint32)
                          for t in ex) for ex in L["experts"]]
    f64 = lambda a: a.view(np.float32).astype(np.float64)
    silu = lambda a: a / (1.0 + np.exp(-a))
    tokens = rng.standard_normal((7, m.hidden))
    top2 = np.stack([rng.permutation(n_exp)[:2] for _ in range(7)])
    gatew = rng.random((7, 2))

    def expert_ffn(g, u, d, x):
        return (silu(x @ g.T) * (x @ u.T)) @ d.T

    want = np.zeros((7, m.hidden))
    for t in range(7):
        for j in range(2):
            g, u, d = (f64(a) for a in L["experts"][top2[t, j]])
            want[t] += gatew[t, j] * expert_ffn(g, u, d, tokens[t])

    src = [moe_shard_of(layers, 2, r, n_exp, 0) for r in range(2)]
    for kp, page in [(4, 0), (8, 4 * 32), (1, 4 * 64)]:
        x = oracle.Moe(n_exp, page, False, bool(page))
        own, first, tensor, slot, layer = oracle.moe_geometry(m, x, bool(page), kp)
        got = np.zeros_like(want)
        for rp in range(kp):
            st, sh = oracle.reshard_weights_moe(m, x, 2, kp, rp, src)
            assert st == oracle.OK
            w = sh.view(np.float32).astype(np.float64)
            for j in range(own):
                ex = rp * own + j
                at = first + j * slot
                g = w[at:at + tensor].reshape(m.ffn_dim, m.hidden)
                u = w[at + tensor:at + 2 * tensor].reshape(m.ffn_dim, m.hidden)
                d = w[at + 2 * tensor:at + 3 * tensor].reshape(m.hidden, m.ffn_dim)
                for t in range(7):
                    for c in range(2):
                        if top2[t, c] == ex:
                            got[t] += gatew[t, c] * expert_ffn(g, u, d, tokens[t])
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_rejects_unsupported_degrees_and_pages():
    layers = moe_full_model(MODEL, E, seed=1)
    src = [moe_shard_of(layers, 1, 0, E, 0)]
    assert oracle.reshard_weights_moe(MODEL, oracle.Moe(E), 1, 5, 0, src)[0] == oracle.ERR_ARG
    assert oracle.reshard_weights_moe(MODEL, oracle.Moe(E), 1, 4, 4, src)[0] == oracle.ERR_ARG
    assert oracle.reshard_weights_moe(MODEL, oracle.Moe(0), 1, 1, 0, src)[0] == oracle.ERR_ARG
    assert oracle.reshard_weights_moe(MODEL, oracle.Moe(E, 63, True, True), 1, 1, 0, src)[0] == \
        oracle.ERR_ARG
    assert oracle.moe_shard_elems(MODEL, oracle.Moe(E), False, 16) == -1
    # a needed source rank that is missing is an error, an unneeded one may be absent
    two = [moe_shard_of(layers, 2, r, E, 0) for r in range(2)]
    assert oracle.reshard_weights_moe(MODEL, oracle.Moe(E), 2, 4, 0, [two[0], None])[0] == oracle.OK
    assert oracle.reshard_weights_moe(MODEL, oracle.Moe(E), 2, 4, 3, [two[0], None])[0] == \
        oracle.ERR_ARG
