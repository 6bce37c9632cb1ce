"""GPU parity for the padded partition-major FFN layout (Sec. 3.2, Improvement 1): building it
from dense shards, gathering partitions between padded shards, and going back to dense, all
through amoeba_reshard_weights, bit for bit against the oracle (zero gaps included)."""
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


def shape(m, pad):
    return ab.ModelShape(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_dim,
                         elem_bytes=m.elem_bytes, w_layout_src=int(pad.src_padded),
                         w_layout_dst=int(pad.dst_padded), pad_max_tp=pad.max_tp,
                         pad_page_bytes=pad.page_bytes)


def sources(m, pad, k, seed):
    dense = [wl.random_bits(oracle.shard_elems(m, k), seed=seed + r, elem_bytes=m.elem_bytes)
             for r in range(k)]
    if not pad.src_padded:
        return dense
    up = oracle.Pad(pad.max_tp, pad.page_bytes, src_padded=False, dst_padded=True)
    return [oracle.reshard_weights_padded(m, up, k, k, r, dense)[1] for r in range(k)]


def check(m, pad, k, kp, rp, src, tune=None):
    st, want = oracle.reshard_weights_padded(m, pad, k, kp, rp, src)
    assert st == oracle.OK
    plan = ab.amoeba_plan(shape(m, pad), k, kp, rp)
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


SMALL = oracle.Model(n_layers=2, hidden=24, n_q_heads=8, n_kv_heads=4, head_dim=4, ffn_dim=72)


@pytest.mark.parametrize("src_padded,dst_padded", [(False, True), (True, True), (True, False)])
@pytest.mark.parametrize("T,page", [(4, 64), (4, 1000), (8, 128), (2, 2)])
def test_padded_small_all_ranks(T, page, src_padded, dst_padded):
    pad = oracle.Pad(T, page, src_padded, dst_padded)
    for k, kp in [(1, 2), (1, 4), (4, 1), (2, 4), (4, 2), (2, 2)]:
        if T % k or T % kp:
            continue
        src = sources(SMALL, pad, k, seed=T + k * 10 + kp)
        for rp in range(kp):
            check(SMALL, pad, k, kp, rp, src)


@pytest.mark.parametrize("elem_bytes", [1, 2, 4])
def test_padded_several_tiles_and_element_widths(elem_bytes):
    """Partitions of 75 KiB at 2-byte elements padded to 16 KiB pages, strided down_proj
    pieces, grid-stride launch."""
    m = oracle.Model(n_layers=3, hidden=320, n_q_heads=8, n_kv_heads=4, head_dim=40, ffn_dim=480,
                     elem_bytes=elem_bytes)
    for sp, dp in [(False, True), (True, True), (True, False)]:
        pad = oracle.Pad(4, 16384, sp, dp)
        for k, kp, rp in [(1, 4, 2), (4, 2, 1), (2, 1, 0)]:
            src = sources(m, pad, k, seed=elem_bytes * 7 + k)
            check(m, pad, k, kp, rp, src)
            check(m, pad, k, kp, rp, src, tune={ab.TUNE_W_GRID: 11, ab.TUNE_W_THREADS: 256,
                                                ab.TUNE_W_UNROLL: 2})


def test_padded_unaligned_partitions_with_2mib_pages():
    """The paper's unaligned example (Table 2, FFN 27648 at TP4) with real 2 MiB pages, at a
    quarter of the hidden size so the per-element oracle finishes in seconds: partitions of
    8.4375 pages padded to 9.  dense TP1 -> padded TP1 (load), padded TP4 -> padded TP2
    (scale-down gather)."""
    m = oracle.Model(n_layers=1, hidden=1280, n_q_heads=8, n_kv_heads=8, head_dim=128,
                     ffn_dim=27648)
    page = 2 << 20
    pad = oracle.Pad(4, page, False, True)
    src = sources(m, pad, 1, seed=3)
    check(m, pad, 1, 1, 0, src)
    pad = oracle.Pad(4, page, True, True)
    src = sources(m, pad, 4, seed=4)
    check(m, pad, 4, 2, 1, src)


def test_moving_only_the_attention_part_or_only_the_ffn_part():
    """amoeba_reshard_weights_part splits one reshard in two disjoint halves: the attention tensors and
    the FFN tensors.  Each half leaves the other half's bytes alone; together they give the
    oracle's shard.  (A padded scale-up uses the attention half only: its FFN is a view.)"""
    m = oracle.Model(n_layers=2, hidden=64, n_q_heads=8, n_kv_heads=4, head_dim=8, ffn_dim=96)
    for pad in (oracle.Pad(4, 256, True, True), oracle.Pad(4, 256, False, False)):
        k, kp, rp = 1, 4, 2
        src = sources(m, pad, k, seed=6)
        if pad.dst_padded:
            st, want = oracle.reshard_weights_padded(m, pad, k, kp, rp, src)
        else:
            st, want = oracle.reshard_weights(m, k, kp, rp, src)
        assert st == oracle.OK
        plan = ab.amoeba_plan(shape(m, pad), k, kp, rp)
        n = ab.amoeba_plan_shard_bytes(plan, 1)
        dev = [to_dev(a) for a in src]
        halves = []
        for part in (ab.PART_ATTENTION, ab.PART_FFN):
            out = torch.full((n,), 0x5C, dtype=torch.uint8, device="cuda")
            ab.amoeba_reshard_weights_part(plan, dev, out, part)
            torch.cuda.synchronize()
            halves.append(out.cpu().numpy())
        a, f = halves
        w = want.view(np.uint8)
        touched_a, touched_f = a != 0x5C, f != 0x5C
        assert not (touched_a & touched_f).any()
        assert (a[touched_a] == w[touched_a]).all() and (f[touched_f] == w[touched_f]).all()
        # bytes neither half changed must be bytes whose value happens to equal the sentinel
        assert (w[~(touched_a | touched_f)] == 0x5C).all()
        layer = n // m.n_layers
        attn_bytes = (8 * 8 // kp + 2 * 4 * 8 // kp) * 64 * 2 + 64 * (8 * 8 // kp) * 2
        first_ffn = np.nonzero(touched_f)[0].min()
        assert np.nonzero(touched_a)[0].max() % layer < first_ffn + layer and first_ffn >= attn_bytes
        plan.close()
