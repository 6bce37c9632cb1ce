"""Host logic for mixture-of-experts plans (Sec. 3.2, EP discussion), no GPU: the planner's
segment table, interpreted with numpy, reproduces the oracle's expert-wise shards byte for
byte, the geometry matches, and the zero-copy view on scale-up is what it claims."""
import numpy as np
import pytest

import oracle
from paper_2509_19729_amd import binding as ab
from moe_helpers import moe_full_model, moe_shard_of
from test_planner_padded import apply_segments

MODEL = oracle.Model(n_layers=2, hidden=12, n_q_heads=24, n_kv_heads=24, head_dim=2, ffn_dim=5,
                     elem_bytes=2)
E = 24


def shape(m, n_experts, page, src_padded, dst_padded):
    return ab.ModelShape(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_dim,
                         elem_bytes=m.elem_bytes, w_layout_src=int(src_padded),
                         w_layout_dst=int(dst_padded), n_experts=n_experts, pad_page_bytes=page)


@pytest.mark.parametrize("page", [64, 1000, 2])
@pytest.mark.parametrize("k,kp", [(1, 1), (1, 4), (4, 1), (2, 8), (8, 2), (2, 3), (3, 2), (6, 4)])
@pytest.mark.parametrize("sp,dp", [(False, False), (False, True), (True, True), (True, False)])
def test_segment_table_reproduces_the_oracle(page, k, kp, sp, dp):
    layers = moe_full_model(MODEL, E, seed=page + 10 * k + kp)
    x = oracle.Moe(E, page, sp, dp)
    src = [moe_shard_of(layers, k, r, E, page // 2 if sp else 0) for r in range(k)]
    for rp in range(kp):
        plan = ab.amoeba_plan(shape(MODEL, E, page, sp, dp), k, kp, rp)
        st, want = oracle.reshard_weights_moe(MODEL, x, k, kp, rp, src)
        assert st == oracle.OK
        assert ab.amoeba_plan_shard_bytes(plan, 1) == want.nbytes
        assert ab.amoeba_plan_shard_bytes(plan, 0) == src[0].nbytes
        got, hits = apply_segments(plan, src, MODEL.n_layers)
        assert (hits == 1).all()                     # every byte, gaps included, written once
        np.testing.assert_array_equal(got.view(np.uint16), want)
        for side, padded, tp in ((0, sp, k), (1, dp, kp)):
            own, first, tensor, slot, layer = oracle.moe_geometry(MODEL, x, padded, tp)
            assert ab.amoeba_plan_expert_info(plan, side) == (own, 2 * first, 2 * tensor, 2 * slot)
            # the generic tensor query points at the first owned expert
            off, rows, cols, layer_elems = ab.amoeba_plan_tensor_info(plan, side, ab.T_DOWN)
            assert (off, rows, cols, layer_elems) == (first + 2 * tensor, MODEL.hidden,
                                                      MODEL.ffn_dim, layer)
            with pytest.raises(ab.AmoebaError):
                ab.amoeba_plan_padded_info(plan, side)
        # whole experts move: the needed source ranks are those whose expert or head range
        # meets the target's
        mask = ab.amoeba_plan_src_rank_mask(plan)
        want_mask = 0
        for s in range(k):
            if s * kp < (rp + 1) * k and rp * k < (s + 1) * kp:
                want_mask |= 1 << s
        assert mask == want_mask


def test_dense_expert_layout_needs_one_segment_per_source_rank():
    """Without gaps a run of whole experts is one contiguous range on both sides."""
    plan = ab.amoeba_plan(shape(MODEL, E, 0, False, False), 8, 2, 1)
    segs = [ab.amoeba_plan_segment(plan, i) for i in range(ab.amoeba_plan_num_segments(plan))]
    ffn = [s for s in segs if s[3] >= ab.amoeba_plan_expert_info(plan, 1)[1]]
    assert len(ffn) == 4 and all(s[5] == 1 for s in ffn)          # 4 source ranks, rows == 1
    assert sorted(s[0] for s in ffn) == [4, 5, 6, 7]


def test_zero_copy_view_on_scale_up():
    layers = moe_full_model(MODEL, E, seed=11)
    for page in (0, 256):
        padded = bool(page)
        x = oracle.Moe(E, page, padded, padded)
        for k, kp in [(1, 4), (2, 8), (1, 3), (4, 4)]:
            src = [moe_shard_of(layers, k, r, E, page // 2) for r in range(k)]
            for rp in range(kp):
                plan = ab.amoeba_plan(shape(MODEL, E, page, padded, padded), k, kp, rp)
                view = ab.amoeba_plan_ffn_view(plan)
                assert view is not None
                rank, off, nbytes, src_layer = view
                assert rank == rp * k // kp and src_layer * MODEL.n_layers == src[0].nbytes
                if page:
                    assert off % page == 0 and nbytes % page == 0
                st, want = oracle.reshard_weights_moe(MODEL, x, k, kp, rp, src)
                own, first, tensor, slot = ab.amoeba_plan_expert_info(plan, 1)
                dst_layer = ab.amoeba_plan_shard_bytes(plan, 1) // MODEL.n_layers
                assert nbytes == dst_layer - first == own * slot
                s = src[rank].view(np.uint8).reshape(MODEL.n_layers, src_layer)
                d = want.view(np.uint8).reshape(MODEL.n_layers, dst_layer)
                np.testing.assert_array_equal(d[:, first:], s[:, off:off + nbytes])
    # no view when scaling down or when the two sides are laid out differently
    assert ab.amoeba_plan_ffn_view(ab.amoeba_plan(shape(MODEL, E, 64, True, True), 4, 2, 0)) is None
    assert ab.amoeba_plan_ffn_view(ab.amoeba_plan(shape(MODEL, E, 64, False, True), 1, 2, 0)) is None


def test_padding_overhead_of_the_papers_moe_shapes():
    """Table 2, MoE rows: an expert of three 2880 x 2880 16-bit projections is 23.73 pages of
    2 MiB and occupies 24: 1.1 % overhead; an expert of the EP experiment's model (three
    768 x 2048 projections, 9 MiB) occupies 10 MiB: 11 %.  Both inside the 0-14 % the paper
    reports (Sec. 4.2.2)."""
    s = ab.ModelShape(1, 2880, 64, 8, 64, 2880, w_layout_src=1, w_layout_dst=1, n_experts=128,
                      pad_page_bytes=2 << 20)
    plan = ab.amoeba_plan(s, 1, 4, 0)
    own, first, tensor, slot = ab.amoeba_plan_expert_info(plan, 1)
    assert own == 32 and tensor == 2880 * 2880 * 2 and slot == 24 * (2 << 20)
    assert (slot - 3 * tensor) / (3 * tensor) == pytest.approx(0.01136, abs=1e-4)
    s = ab.ModelShape(1, 2048, 32, 4, 128, 768, w_layout_src=1, w_layout_dst=1, n_experts=128,
                      pad_page_bytes=2 << 20)
    own, first, tensor, slot = ab.amoeba_plan_expert_info(ab.amoeba_plan(s, 1, 4, 0), 1)
    assert (slot - 3 * tensor) / (3 * tensor) == pytest.approx(1 / 9)


def test_rejects_bad_expert_parameters():
    for k, kp, kw in [(1, 5, {}), (16, 1, {}), (1, 2, dict(n_experts=-1)),
                      (1, 2, dict(w_layout_dst=1, pad_page_bytes=3)),
                      (1, 2, dict(w_layout_dst=1, pad_page_bytes=0))]:
        args = dict(n_experts=E)
        args.update(kw)
        with pytest.raises(ab.AmoebaError):
            ab.amoeba_plan(ab.ModelShape(2, 12, 24, 24, 2, 5, **args), k, kp, 0)
    # the degree need not divide one expert's intermediate size
    assert ab.amoeba_plan(ab.ModelShape(2, 12, 24, 24, 2, 5, n_experts=E), 2, 4, 1) is not None
    plan = ab.amoeba_plan(ab.ModelShape(2, 12, 24, 24, 2, 5), 1, 1, 0)
    with pytest.raises(ab.AmoebaError):
        ab.amoeba_plan_expert_info(plan, 0)
