"""Host logic for the padded FFN layout (Sec. 3.2, Improvement 1), no GPU: the planner's
segment table, interpreted with numpy, reproduces the oracle's padded shards byte for byte
(zero gaps included), the geometry matches, and the zero-copy view is what it claims."""
import numpy as np
import pytest

import oracle
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl

MODEL = oracle.Model(n_layers=2, hidden=24, n_q_heads=8, n_kv_heads=4, head_dim=4, ffn_dim=72,
                     elem_bytes=2)


def shape(m, T, page, src_padded, dst_padded):
    return ab.ModelShape(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_dim,
                         elem_bytes=m.elem_bytes, w_layout_src=int(src_padded),
                         w_layout_dst=int(dst_padded), pad_max_tp=T, pad_page_bytes=page)


def apply_segments(plan, src_shards, n_layers):
    src_layer = ab.amoeba_plan_shard_bytes(plan, 0) // n_layers
    dst_layer = ab.amoeba_plan_shard_bytes(plan, 1) // n_layers
    dst = np.full(dst_layer * n_layers, 0xEE, dtype=np.uint8)
    hits = np.zeros(dst_layer * n_layers, dtype=np.uint8)
    for idx in range(ab.amoeba_plan_num_segments(plan)):
        r, so, sp, do, dp, rows, run = ab.amoeba_plan_segment(plan, idx)
        for l in range(n_layers):
            for row in range(rows):
                b = l * dst_layer + do + row * dp
                if r < 0:
                    dst[b:b + run] = 0
                else:
                    a = l * src_layer + so + row * sp
                    dst[b:b + run] = src_shards[r].view(np.uint8)[a:a + run]
                hits[b:b + run] += 1
    return dst, hits


def source_shards(m, pad, k, seed):
    """Padded sources are produced by the oracle from random dense shards (so their gaps hold
    zeros, as the layout requires)."""
    dense = [wl.random_bits(oracle.shard_elems(m, k), seed=seed + r) for r in range(k)]
    if not pad.src_padded:
        return dense
    to_padded = oracle.Pad(pad.max_tp, pad.page_bytes, src_padded=False, dst_padded=True)
    return [oracle.reshard_weights_padded(m, to_padded, k, k, r, dense)[1] for r in range(k)]


@pytest.mark.parametrize("T,page", [(4, 64), (4, 1000), (8, 128), (2, 2)])
@pytest.mark.parametrize("k,kp", [(1, 1), (1, 2), (1, 4), (4, 1), (2, 4), (4, 2), (2, 2)])
@pytest.mark.parametrize("src_padded,dst_padded", [(False, True), (True, True), (True, False)])
def test_segment_table_reproduces_the_oracle(T, page, k, kp, src_padded, dst_padded):
    if T % k or T % kp:
        with pytest.raises(ab.AmoebaError):
            ab.amoeba_plan(shape(MODEL, T, page, src_padded, dst_padded), k, kp, 0)
        return
    pad = oracle.Pad(T, page, src_padded, dst_padded)
    src = source_shards(MODEL, pad, k, seed=T * 100 + k * 10 + kp)
    for rp in range(kp):
        plan = ab.amoeba_plan(shape(MODEL, T, page, src_padded, dst_padded), k, kp, rp)
        st, want = oracle.reshard_weights_padded(MODEL, pad, k, kp, rp, src)
        assert st == oracle.OK
        assert ab.amoeba_plan_shard_bytes(plan, 1) == want.nbytes
        assert ab.amoeba_plan_shard_bytes(plan, 0) == src[0].nbytes
        got, hits = apply_segments(plan, src, MODEL.n_layers)
        assert (hits == 1).all()                     # every byte, gaps included, written once
        np.testing.assert_array_equal(got.view(np.uint16), want)
        for side, padded, tp in ((0, src_padded, k), (1, dst_padded, kp)):
            if padded:
                info = ab.amoeba_plan_padded_info(plan, side)
                assert info == tuple(2 * x for x in oracle.padded_geometry(MODEL, pad, tp))
                assert info[1] % page == 0 and info[3] % page == 0 and info[5] % page == 0
            else:
                with pytest.raises(ab.AmoebaError):
                    ab.amoeba_plan_padded_info(plan, side)


def test_zero_copy_view_on_scale_up():
    T, page = 4, 256
    pad = oracle.Pad(T, page, True, True)
    for k, kp in [(1, 2), (1, 4), (2, 4), (2, 2)]:
        src = source_shards(MODEL, pad, k, seed=k + kp)
        for rp in range(kp):
            plan = ab.amoeba_plan(shape(MODEL, T, page, True, True), k, kp, rp)
            view = ab.amoeba_plan_ffn_view(plan)
            assert view is not None
            rank, off, nbytes, src_layer = view
            assert rank == rp * k // kp and off % page == 0 and nbytes % page == 0
            st, want = oracle.reshard_weights_padded(MODEL, pad, k, kp, rp, src)
            _, attn_padded, _, _, _, dst_layer = ab.amoeba_plan_padded_info(plan, 1)
            assert nbytes == dst_layer - attn_padded and src_layer * MODEL.n_layers == src[0].nbytes
            s = src[rank].view(np.uint8).reshape(MODEL.n_layers, src_layer)
            d = want.view(np.uint8).reshape(MODEL.n_layers, dst_layer)
            np.testing.assert_array_equal(d[:, attn_padded:], s[:, off:off + nbytes])
    # no view when scaling down, or when a side is dense
    assert ab.amoeba_plan_ffn_view(ab.amoeba_plan(shape(MODEL, T, page, True, True), 4, 2, 0)) is None
    assert ab.amoeba_plan_ffn_view(ab.amoeba_plan(shape(MODEL, T, page, False, True), 1, 2, 0)) is None


def test_padding_overhead_at_the_papers_model_shapes():
    """Sec. 4.2.2 reports 0-14 % memory overhead from padding; for the dense models of
    Table 2 with T = 4 and 2 MiB pages it is 0 % (Llama-3.1-70B) and 0.74 % (Qwen2.5-32B)."""
    for hidden, ffn, want in [(8192, 28672, 0.0), (5120, 27648, 0.25 / 33.75)]:
        s = ab.ModelShape(1, hidden, 64, 8, 128, ffn, w_layout_src=1, w_layout_dst=1,
                          pad_max_tp=4, pad_page_bytes=2 << 20)
        plan = ab.amoeba_plan(s, 1, 4, 0)
        _, _, part, part_padded, _, _ = ab.amoeba_plan_padded_info(plan, 1)
        assert (part_padded - part) / part == pytest.approx(want, abs=1e-9)


def test_rejects_bad_padding_parameters():
    for kw in (dict(pad_max_tp=5), dict(pad_max_tp=0), dict(pad_page_bytes=3),
               dict(pad_page_bytes=0), dict(pad_max_tp=32)):
        args = dict(pad_max_tp=4, pad_page_bytes=64)
        args.update(kw)
        s = ab.ModelShape(2, 24, 8, 4, 4, 72, w_layout_dst=1, **args)
        with pytest.raises(ab.AmoebaError):
            ab.amoeba_plan(s, 1, 2, 0)
    with pytest.raises(ab.AmoebaError):
        ab.amoeba_plan(ab.ModelShape(2, 24, 8, 4, 4, 72, w_layout_dst=2, pad_max_tp=4,
                                     pad_page_bytes=64), 1, 2, 0)
