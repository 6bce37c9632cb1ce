"""The reshard calls under HIP graph capture: they enqueue kernels only (no allocation, no
memset node, no synchronisation), so a serving loop can record them once and replay.
Every replay is checked against the eager result, with eager work between replays."""
import sys

import numpy as np
import pytest
import torch

import oracle
from gpu_util import model_for_kv, shape_from, to_dev
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    sys.stdout.flush()
    yield


@pytest.mark.parametrize("static", [False, True])
@pytest.mark.parametrize("three_kernels", [False, True])
def test_weights_and_kv_replay_from_a_captured_graph(static, three_kernels):
    """static: the KV call is the entry point that allocates nothing (its reason to exist is code
    under capture).  three_kernels: the scan / table / regroup path instead of the one-launch path
    this small table would take."""
    B, d, H, layers = 16, 64, 8, 3
    lens0 = np.array([40, 100, 7, 33, 0, 16], dtype=np.int32)
    nb = (lens0.astype(np.int64) + B - 1) // B
    P = int(nb.sum()) + 9
    W = int(nb.max()) + 2
    rng = np.random.default_rng(5)
    ids = rng.permutation(P)[:int(nb.sum())]
    table = np.full((len(lens0), W), -1, dtype=np.int32)
    p = 0
    for i, n in enumerate(nb):
        table[i, :n] = ids[p:p + n]
        p += int(n)
    kv = oracle.KV(kv_layers=layers, n_kv_heads=H, head_dim=d, block_tokens=B,
                   num_seqs=len(lens0), max_blocks_per_seq=W, src_pool_blocks=P,
                   dst_pool_blocks=int(nb.sum()) + 3)
    m = model_for_kv(kv)
    k, kp, rp = 2, 1, 0
    plan = ab.amoeba_plan(shape_from(m, kv), k, kp, rp)
    if three_kernels:
        ab.amoeba_plan_tune(plan, ab.TUNE_KV_SMALL_TABLE, 1)
    reshard_kv = ab.amoeba_reshard_kv_static if static else ab.amoeba_reshard_kv

    n_src = oracle.shard_elems(m, k)
    w_src_np = [wl.random_bits(n_src, seed=70 + s) for s in range(k)]
    be = oracle.kv_block_elems(kv, k)
    pools_np = [wl.random_bits(layers * P * be, seed=80 + s).reshape(layers, P, be)
                for s in range(k)]
    w_src = [to_dev(a) for a in w_src_np]
    pools = [to_dev(a) for a in pools_np]
    w_dst = torch.zeros(ab.amoeba_plan_shard_bytes(plan, 1) // 2, dtype=torch.int16, device="cuda")
    bd = ab.amoeba_plan_kv_block_bytes(plan, 1) // 2
    kv_dst = torch.zeros((layers, kv.dst_pool_blocks, bd), dtype=torch.int16, device="cuda")
    table_d = torch.from_numpy(table).cuda()
    lens_d = torch.from_numpy(lens0).cuda()
    out_table = torch.zeros((len(lens0), W), dtype=torch.int32, device="cuda")

    def expect(lens):
        st, want_w = oracle.reshard_weights(m, k, kp, rp, w_src_np)
        assert st == oracle.OK
        pool = np.zeros((layers, kv.dst_pool_blocks, bd), dtype=np.uint16)
        st, t, _ = oracle.reshard_kv(kv, k, kp, rp, pools_np, table, lens, pool)
        assert st == oracle.OK
        return want_w, pool, t

    # warm up on a side stream (first launches load code objects), then capture
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ab.amoeba_reshard_weights(plan, w_src, w_dst)
        reshard_kv(plan, pools, table_d, lens_d, kv_dst, out_table)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ab.amoeba_reshard_weights(plan, w_src, w_dst)
        reshard_kv(plan, pools, table_d, lens_d, kv_dst, out_table)

    for it in range(4):
        # eager work between replays: wipe the outputs and change the lengths in place, so a
        # replay that reused stale results or stale tables would be caught
        lens = lens0.copy()
        lens[it % len(lens)] = max(0, int(lens[it % len(lens)]) - 5 * it)
        lens_d.copy_(torch.from_numpy(lens))
        w_dst.zero_()
        kv_dst.zero_()
        out_table.fill_(-5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_w, want_pool, want_t = expect(lens)
        np.testing.assert_array_equal(w_dst.cpu().numpy().view(np.uint16), want_w)
        np.testing.assert_array_equal(out_table.cpu().numpy(), want_t)
        np.testing.assert_array_equal(kv_dst.cpu().numpy().view(np.uint16), want_pool)
        rc, total = ab.amoeba_kv_status(plan)      # outside the graph: it synchronises
        assert rc == ab.OK and total == int(((lens.astype(np.int64) + B - 1) // B).sum())
    plan.close()


def test_inplace_merge_replays_from_a_captured_graph():
    """The in-place merge clears its flags with a kernel (no memset node) and compacts its work
    list on the device, so it can be captured too.  The pool is restored and the lengths are
    changed eagerly between replays; every replay must match the oracle."""
    from test_gpu_merge import instances

    m, k, rp = 2, 1, 1
    lens0 = [[33, 7, 100], [64, 1, 18]]
    cfg, insts = instances(m, k, lens0, n_heads=4, d=64, B=16, layers=2, P=16, W=9, seed=3)
    g = rp % m
    plan = ab.amoeba_plan(shape_from(model_for_kv(cfg), cfg), k, k * m, rp)
    pristine = to_dev(insts[g]["pools"][0])
    local = pristine.clone()
    remote = [None if g2 == g else to_dev(insts[g2]["pools"][0]) for g2 in range(m)]
    tabs = [torch.from_numpy(i["table"]).cuda() for i in insts]
    lens_d = [torch.from_numpy(i["lens"]).cuda() for i in insts]
    out_table = torch.zeros((m * cfg.num_seqs, cfg.max_blocks_per_seq), dtype=torch.int32,
                            device="cuda")

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ab.amoeba_merge_kv_inplace(plan, local, remote, tabs, lens_d, out_table)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ab.amoeba_merge_kv_inplace(plan, local, remote, tabs, lens_d, out_table)

    for it in range(4):
        lens = [i["lens"].copy() for i in insts]
        lens[it % m][it % 3] = max(0, int(lens[it % m][it % 3]) - 9 * it)
        for dev, host in zip(lens_d, lens):
            dev.copy_(torch.from_numpy(host))
        local.copy_(pristine)
        out_table.fill_(-5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_pool = insts[g]["pools"][0].copy()
        st, want_table, want_n = oracle.merge_kv_inplace(
            cfg, k, m, rp, want_pool,
            [None if g2 == g else insts[g2]["pools"][0] for g2 in range(m)],
            [i["table"] for i in insts], lens)
        assert st == oracle.OK
        np.testing.assert_array_equal(out_table.cpu().numpy(), want_table)
        np.testing.assert_array_equal(
            local.cpu().numpy().view(want_pool.dtype).reshape(want_pool.shape), want_pool)
        rc, n = ab.amoeba_merge_kv_status(plan)
        assert rc == ab.OK and n == want_n
    plan.close()
