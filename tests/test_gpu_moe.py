"""GPU parity for mixture-of-experts plans (Sec. 3.2, EP discussion; TPkEPk of Sec. 4.3):
attention tensors re-sliced by head, whole experts gathered by rank, with and without page
padding, through amoeba_reshard_weights, bit for bit against the oracle."""
import sys

import numpy as np
import pytest
import torch

import oracle
from gpu_util import to_dev
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    sys.stdout.flush()
    yield


def shape(m, x):
    return ab.ModelShape(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_dim,
                         elem_bytes=m.elem_bytes, w_layout_src=int(x.src_padded),
                         w_layout_dst=int(x.dst_padded), n_experts=x.n_experts,
                         pad_page_bytes=x.page_bytes)


def sources(m, x, k, seed):
    """Random dense expert-wise shards; padded sources are made from them by the oracle (k -> k,
    every rank) so that their gaps hold zeros."""
    flat = oracle.Moe(x.n_experts)
    dense = [wl.random_bits(oracle.moe_shard_elems(m, flat, False, k), seed=seed + r,
                            elem_bytes=m.elem_bytes) for r in range(k)]
    if not x.src_padded:
        return dense
    up = oracle.Moe(x.n_experts, x.page_bytes, False, True)
    return [oracle.reshard_weights_moe(m, up, k, k, r, dense)[1] for r in range(k)]


def check(m, x, k, kp, rp, src, tune=None):
    st, want = oracle.reshard_weights_moe(m, x, k, kp, rp, src)
    assert st == oracle.OK
    plan = ab.amoeba_plan(shape(m, x), k, kp, rp)
    for knob, val in (tune or {}).items():
        ab.amoeba_plan_tune(plan, knob, val)
    n = ab.amoeba_plan_shard_bytes(plan, 1)
    assert n == want.nbytes
    mask = ab.amoeba_plan_src_rank_mask(plan)
    dev = [to_dev(a) if mask >> r & 1 else None for r, a in enumerate(src)]
    guard = 512
    buf = torch.full((n + 2 * guard,), 0x5C, dtype=torch.uint8, device="cuda")
    ab.amoeba_reshard_weights(plan, dev, buf[guard:guard + n])
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[:guard] == 0x5C).all() and (host[guard + n:] == 0x5C).all()
    np.testing.assert_array_equal(host[guard:guard + n].view(want.dtype), want)
    plan.close()


SMALL = oracle.Model(n_layers=2, hidden=12, n_q_heads=24, n_kv_heads=24, head_dim=2, ffn_dim=5)


@pytest.mark.parametrize("sp,dp", [(False, False), (False, True), (True, True), (True, False)])
@pytest.mark.parametrize("page", [64, 1000, 2])
def test_moe_small_all_ranks(page, sp, dp):
    """24 experts of 5 x 12 (odd sizes: 2-byte vectors), every rank of several degree pairs,
    non-multiples included."""
    x = oracle.Moe(24, page, sp, dp)
    for k, kp in [(1, 4), (4, 1), (2, 8), (8, 2), (2, 3), (3, 2), (6, 4)]:
        src = sources(SMALL, x, k, seed=page + k * 10 + kp)
        for rp in range(kp):
            check(SMALL, x, k, kp, rp, src)


@pytest.mark.parametrize("elem_bytes", [1, 2, 4])
def test_moe_several_tiles_and_element_widths(elem_bytes):
    """16 experts of 48 x 320: experts of 90 KiB at 2-byte elements padded to 16 KiB pages (six
    pages each, ragged last tile), one-tile-per-workgroup and grid-stride launches."""
    m = oracle.Model(n_layers=3, hidden=320, n_q_heads=8, n_kv_heads=4, head_dim=40, ffn_dim=48,
                     elem_bytes=elem_bytes)
    for sp, dp in [(False, False), (False, True), (True, True), (True, False)]:
        x = oracle.Moe(16, 16384, sp, dp)
        for k, kp, rp in [(1, 4, 2), (4, 2, 1), (2, 1, 0)]:
            src = sources(m, x, k, seed=elem_bytes * 7 + k)
            check(m, x, k, kp, rp, src)
            check(m, x, k, kp, rp, src, tune={ab.TUNE_W_GRID: 11, ab.TUNE_W_THREADS: 256,
                                              ab.TUNE_W_UNROLL: 2})


def test_moe_real_expert_shape_with_2mib_pages():
    """One layer of the paper's EP experiment at real expert size (three 768 x 2048
    projections, 9 MiB -> 5 pages of 2 MiB) with 16 of the 128 experts so the oracle finishes in
    seconds: dense -> padded (load), padded EP4 -> padded EP1 (scale-down gather), padded EP1
    -> EP4 (scale-up; the FFN part is also checked to be the promised view)."""
    m = oracle.Model(n_layers=1, hidden=2048, n_q_heads=32, n_kv_heads=4, head_dim=128,
                     ffn_dim=768)
    page = 2 << 20
    x = oracle.Moe(16, page, False, True)
    check(m, x, 1, 1, 0, sources(m, x, 1, seed=3))
    x = oracle.Moe(16, page, True, True)
    check(m, x, 4, 1, 0, sources(m, x, 4, seed=4))
    src = sources(m, x, 1, seed=5)
    check(m, x, 1, 4, 1, src)
    plan = ab.amoeba_plan(shape(m, x), 1, 4, 1)
    rank, off, nbytes, src_layer = ab.amoeba_plan_ffn_view(plan)
    own, first, tensor, slot = ab.amoeba_plan_expert_info(plan, 1)
    st, want = oracle.reshard_weights_moe(m, x, 1, 4, 1, src)
    assert rank == 0 and off % page == 0 and nbytes == own * slot
    np.testing.assert_array_equal(want.view(np.uint8)[first:first + nbytes],
                                  src[0].view(np.uint8)[off:off + nbytes])
    plan.close()


def test_moe_attention_half_only_for_a_scale_up():
    """A scale-up whose experts stay where they are (zero-copy view) moves only the attention
    tensors: with AMOEBA_PART_ATTENTION the expert part of the target is not written."""
    m = oracle.Model(n_layers=2, hidden=64, n_q_heads=8, n_kv_heads=4, head_dim=8, ffn_dim=24)
    x = oracle.Moe(8, 256, True, True)
    src = sources(m, x, 1, seed=8)
    st, want = oracle.reshard_weights_moe(m, x, 1, 4, 3, src)
    plan = ab.amoeba_plan(shape(m, x), 1, 4, 3)
    n = ab.amoeba_plan_shard_bytes(plan, 1)
    own, first, tensor, slot = ab.amoeba_plan_expert_info(plan, 1)
    out = torch.full((n,), 0x5C, dtype=torch.uint8, device="cuda")
    ab.amoeba_reshard_weights_part(plan, [to_dev(src[0])], out, ab.PART_ATTENTION)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(m.n_layers, -1)
    w = want.view(np.uint8).reshape(m.n_layers, -1)
    np.testing.assert_array_equal(got[:, :first], w[:, :first])
    assert (got[:, first:] == 0x5C).all()
    plan.close()
