"""amoeba_reshard_kv_static(): the entry point that allocates nothing (its kernels' workspace
is a static device array) against amoeba_reshard_kv() on the same inputs, through the C ABI,
bit for bit: two calls in a row, the second with a smaller input, so that what the first call
left in the shared array must not leak into the second."""
import sys

import numpy as np
import pytest
import torch

import oracle
from gpu_util import model_for_kv, shape_from, to_dev
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl

pytestmark = pytest.mark.gpu

HM, TM = ab.KV_HEAD_MAJOR, ab.KV_TOKEN_MAJOR


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    sys.stdout.flush()
    yield


def case(k, lens, lay_s, lay_d, n_heads, d, B, layers, seed, slack=3):
    lens = np.asarray(lens, dtype=np.int32)
    nb = (np.maximum(lens, 0).astype(np.int64) + B - 1) // B
    P = int(nb.sum()) + 5
    rng = np.random.default_rng(seed)
    ids = rng.permutation(P)[:int(nb.sum())]
    W = max(1, int(nb.max(initial=0))) + 2
    table = np.full((len(lens), W), -1, dtype=np.int32)
    p = 0
    for i, n in enumerate(nb):
        table[i, :n] = ids[p:p + n]
        p += int(n)
    cfg = oracle.KV(kv_layers=layers, n_kv_heads=n_heads, head_dim=d, block_tokens=B,
                    num_seqs=len(lens), max_blocks_per_seq=W, src_pool_blocks=P,
                    dst_pool_blocks=int(nb.sum()) + slack, layout_src=lay_s, layout_dst=lay_d)
    be = oracle.kv_block_elems(cfg, k)
    pools = [wl.random_bits(layers * P * be, seed=seed * 17 + s).reshape(layers, P, be)
             for s in range(k)]
    return cfg, pools, table, lens


def run_both(cfg, k, kp, rp, pools, table, lens, tune=None):
    """Returns what the two entry points produce for one input: (status, total, table, pool
    bytes with guard bands) each."""
    plan = ab.amoeba_plan(shape_from(model_for_kv(cfg), cfg), k, kp, rp)
    for knob, val in (tune or {}).items():
        ab.amoeba_plan_tune(plan, knob, val)
    n_bytes = cfg.kv_layers * cfg.dst_pool_blocks * ab.amoeba_plan_kv_block_bytes(plan, 1)
    src_dev = [to_dev(a) for a in pools]
    table_dev, lens_dev = torch.from_numpy(table).cuda(), torch.from_numpy(lens).cuda()
    out = []
    for call in (ab.amoeba_reshard_kv, ab.amoeba_reshard_kv_static):
        buf = torch.full((n_bytes + 2048,), 0xA7, dtype=torch.uint8, device="cuda")
        new_table = torch.full(table.shape, -9, dtype=torch.int32, device="cuda")
        call(plan, src_dev, table_dev, lens_dev, buf[1024:1024 + n_bytes], new_table)
        st, total = ab.amoeba_kv_status(plan)
        out.append((st, total, new_table.cpu().numpy(), buf.cpu().numpy()))
    plan.close()
    return out


def same(a, b):
    assert a[0] == b[0] and a[1] == b[1]
    np.testing.assert_array_equal(a[2], b[2])
    np.testing.assert_array_equal(a[3], b[3])


@pytest.mark.parametrize("tune", [None, {ab.TUNE_KV_SMALL_TABLE: 1}])
@pytest.mark.parametrize("lay_s,lay_d", [(HM, HM), (TM, HM)])
def test_static_workspace_matches_the_allocating_entry_point_twice_in_a_row(lay_s, lay_d, tune):
    # first call: 70 sequences, 40 KiB blocks, 3 layers (the three-kernel path; d = 64
    # converting goes through the LDS-staged kernel)
    rng = np.random.default_rng(7)
    big = case(2, rng.integers(0, 200, size=70), lay_s, lay_d, n_heads=10, d=64, B=16, layers=3,
               seed=1)
    first = run_both(big[0], 2, 1, 0, *big[1:], tune=tune)
    same(*first)
    assert first[0][0] == ab.OK and first[0][1] > 0
    # second call: fewer and shorter sequences, another geometry (a small table: one launch,
    # unless the three-kernel path is forced)
    small = case(1, [13, 1, 8, 0, 22], lay_s, lay_d, n_heads=8, d=8, B=4, layers=2, seed=2)
    second = run_both(small[0], 1, 2, 1, *small[1:], tune=tune)
    same(*second)
    assert second[0][0] == ab.OK and 0 < second[0][1] < first[0][1]
    # against the oracle as well
    cfg, pools, table, lens = small
    be = oracle.kv_block_elems(cfg, 2)
    want = np.full((cfg.kv_layers, cfg.dst_pool_blocks, be), 0xA7A7, dtype=np.uint16)
    ost, want_table, want_total = oracle.reshard_kv(cfg, 1, 2, 1, pools, table, lens, want)
    assert ost == oracle.OK and want_total == second[1][1]
    np.testing.assert_array_equal(second[1][2], want_table)
    np.testing.assert_array_equal(second[1][3][1024:-1024].view(np.uint16), want.ravel())


def test_static_workspace_reports_errors_like_the_allocating_entry_point():
    cfg, pools, table, lens = case(1, [9, 6, 30], HM, HM, n_heads=4, d=8, B=4, layers=2, seed=3)
    bad = lens.copy()
    bad[1] = -1
    r = run_both(cfg, 1, 2, 0, pools, table, bad)
    same(*r)
    assert r[1][0] == ab.ERR_OVERFLOW
    worse = table.copy()
    worse[2, 1] = cfg.src_pool_blocks + 1
    r = run_both(cfg, 1, 2, 0, pools, worse, lens)
    same(*r)
    assert r[1][0] == ab.ERR_BLOCK_ID
    same(*run_both(cfg, 1, 2, 0, pools, table, lens))      # and the status resets


def test_static_workspace_refuses_what_does_not_fit():
    """2^20 int32 words: a pool of a million blocks does not fit; nothing is launched."""
    kv = oracle.KV(kv_layers=1, n_kv_heads=2, head_dim=8, block_tokens=4, num_seqs=4,
                   max_blocks_per_seq=8, src_pool_blocks=16, dst_pool_blocks=(1 << 20) - 11)
    plan = ab.amoeba_plan(shape_from(model_for_kv(kv), kv), 1, 2, 0)
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    rc = ab.amoeba_reshard_kv_static(plan, [t], t, t, t, t, check=False)
    assert rc == ab.ERR_INVALID_ARG and "static workspace" in ab.amoeba_last_error()
    plan.close()
