"""GPU parity of the in-place instance merge (amoeba_merge_kv_inplace) against the oracle:
the whole local pool (moved and untouched bytes alike), the merged table and the status,
bit for bit."""
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


def instances(m, k, lens_per_inst, n_heads, d, B, layers, P, W, seed, elem_bytes=2):
    """Random pools and tables for m instances at TP=k (rank s of instance g: pools[g][s])."""
    cfg = oracle.KV(kv_layers=layers, n_kv_heads=n_heads, head_dim=d, block_tokens=B,
                    num_seqs=len(lens_per_inst[0]), max_blocks_per_seq=W, src_pool_blocks=P,
                    dst_pool_blocks=P * m, elem_bytes=elem_bytes)
    be = oracle.kv_block_elems(cfg, k)
    out = []
    for g in range(m):
        lens = np.asarray(lens_per_inst[g], dtype=np.int32)
        nb = (np.maximum(lens, 0).astype(np.int64) + B - 1) // B
        rng = np.random.default_rng(seed * 31 + g)
        ids = rng.permutation(P)[:int(nb.sum())]
        table = np.full((len(lens), W), -1, dtype=np.int32)
        p = 0
        for i, n in enumerate(nb):
            table[i, :n] = ids[p:p + n]
            p += int(n)
        pools = [wl.random_bits(layers * P * be, seed=seed * 100 + g * 10 + s,
                                elem_bytes=elem_bytes).reshape(layers, P, be) for s in range(k)]
        out.append(dict(lens=lens, table=table, pools=pools))
    return cfg, out


def check_merge(cfg, insts, m, k, rp, expect=oracle.OK, tune=None):
    s, g = rp // m, rp % m
    tabs, lens = [i["table"] for i in insts], [i["lens"] for i in insts]
    want_pool = insts[g]["pools"][s].copy()
    remote = [None if g2 == g else insts[g2]["pools"][s] for g2 in range(m)]
    ost, want_table, want_n = oracle.merge_kv_inplace(cfg, k, m, rp, want_pool, remote, tabs, lens)
    assert ost == expect

    plan = ab.amoeba_plan(shape_from(model_for_kv(cfg), cfg), k, k * m, rp)
    assert ab.amoeba_plan_merge_factor(plan) == m
    for knob, val in (tune or {}).items():
        ab.amoeba_plan_tune(plan, knob, val)
    guard = 4096
    raw = insts[g]["pools"][s].view(np.uint8).ravel()
    buf = torch.full((raw.size + 2 * guard,), 0xA7, dtype=torch.uint8, device="cuda")
    buf[guard:guard + raw.size] = torch.from_numpy(raw).cuda()
    local = buf[guard:guard + raw.size]
    remote_dev = [None if a is None else to_dev(a) for a in remote]
    tabs_dev = [torch.from_numpy(t).cuda() for t in tabs]
    lens_dev = [torch.from_numpy(x).cuda() for x in lens]
    out_table = torch.full((m * cfg.num_seqs, cfg.max_blocks_per_seq), -9, dtype=torch.int32,
                           device="cuda")
    ab.amoeba_merge_kv_inplace(plan, local, remote_dev, tabs_dev, lens_dev, out_table)
    st, n = ab.amoeba_merge_kv_status(plan)
    code = {oracle.OK: ab.OK, oracle.ERR_OVERFLOW: ab.ERR_OVERFLOW,
            oracle.ERR_BLOCK_ID: ab.ERR_BLOCK_ID}[ost]
    assert st == code and n == want_n
    host = buf.cpu().numpy()
    assert (host[:guard] == 0xA7).all() and (host[guard + raw.size:] == 0xA7).all()
    np.testing.assert_array_equal(out_table.cpu().numpy(), want_table)
    got = host[guard:guard + raw.size].view(want_pool.dtype).reshape(want_pool.shape)
    np.testing.assert_array_equal(got, want_pool)
    plan.close()


LENS4 = [[13, 1, 8, 0, 40], [5, 22, 3, 9, 0], [16, 2, 7, 7, 1], [1, 1, 30, 4, 12]]


@pytest.mark.parametrize("m,k,n_heads", [(4, 1, 8), (2, 1, 8), (2, 2, 8), (3, 2, 12), (2, 4, 16)])
def test_merge_small_every_target_rank(m, k, n_heads):
    cfg, insts = instances(m, k, LENS4[:m], n_heads=n_heads, d=8, B=4, layers=3, P=40, W=14,
                           seed=m * 7 + k)
    for rp in range(k * m):
        check_merge(cfg, insts, m, k, rp)


@pytest.mark.parametrize("elem_bytes,d", [(2, 64), (1, 16), (4, 4), (2, 4), (2, 2), (2, 1), (1, 1)])
def test_merge_every_vector_width_and_several_tiles(elem_bytes, d):
    """d = 64 at 16 bits: sub-blocks of 16 KiB = 16 tiles per block; the small d cases fall
    back to 8/4/2/1-byte accesses."""
    cfg, insts = instances(2, 1, [[33, 7, 100], [64, 1, 18]], n_heads=4, d=d, B=16, layers=2,
                           P=16, W=9, seed=d, elem_bytes=elem_bytes)
    for rp in range(2):
        check_merge(cfg, insts, 2, 1, rp)
    check_merge(cfg, insts, 2, 1, 1, tune={ab.TUNE_KV_GRID: 3, ab.TUNE_NONTEMPORAL: 2})
    # launch shapes: one or four wavefronts per workgroup, grid bounded by a hint that is
    # too small (workgroups stride), exact, or absent (grid covers the pool's capacity)
    for threads, hint in [(64, 1), (256, 1), (64, 9), (256, 9), (0, 0), (0, 9), (256, 0)]:
        check_merge(cfg, insts, 2, 1, 0,
                    tune={ab.TUNE_KV_THREADS: threads, ab.TUNE_KV_BLOCKS_HINT: hint})


def test_merge_degenerate_and_error_cases():
    cfg, insts = instances(2, 1, [[0, 0], [0, 0]], n_heads=4, d=8, B=4, layers=1, P=8, W=4, seed=1)
    check_merge(cfg, insts, 2, 1, 0)                       # nothing to move
    cfg, insts = instances(2, 1, [[9, 4], [5, 8]], n_heads=4, d=8, B=4, layers=2, P=8, W=4, seed=2)
    insts[1]["lens"][0] = -3
    check_merge(cfg, insts, 2, 1, 0, expect=oracle.ERR_OVERFLOW)
    insts[1]["lens"][0] = 5
    check_merge(cfg, insts, 2, 1, 0)                       # the flags reset between calls
    insts[0]["lens"][1] = 4 * 4 + 1                        # needs 5 blocks, the row holds 4
    check_merge(cfg, insts, 2, 1, 1, expect=oracle.ERR_OVERFLOW)
    insts[0]["lens"][1] = 4
    insts[1]["table"][1, 0] = 8                            # one past the pool
    check_merge(cfg, insts, 2, 1, 0, expect=oracle.ERR_BLOCK_ID)
    insts[0]["table"][0, 1] = -2                           # a bad id in the local table
    check_merge(cfg, insts, 2, 1, 0, expect=oracle.ERR_BLOCK_ID)


def test_merge_shared_block_ids_and_a_bad_id_count_slots_once():
    """Two sequences of one instance share a block (a common prefix) and another cell holds
    an id outside the pool: the table carries the shared id twice, the slot is filled and
    counted once, the bad cell reads -1 and is not counted (the oracle's count is pinned on
    the CPU from the input tables alone)."""
    cfg, insts = instances(3, 1, [[13, 8, 9], [5, 22, 6], [16, 2, 7]], n_heads=6, d=8, B=4,
                           layers=2, P=24, W=8, seed=21)
    insts[1]["table"][2, 0] = insts[1]["table"][0, 0]
    insts[1]["table"][2, 1] = insts[1]["table"][0, 1]
    for rp in range(3):
        check_merge(cfg, insts, 3, 1, rp)
    insts[2]["table"][0, 1] = 24 + 3
    for rp in range(3):
        check_merge(cfg, insts, 3, 1, rp, expect=oracle.ERR_BLOCK_ID)


def test_merge_rejects_plans_that_do_not_qualify():
    kv = oracle.KV(kv_layers=1, n_kv_heads=8, head_dim=8, block_tokens=4, num_seqs=2,
                   max_blocks_per_seq=4, src_pool_blocks=8, dst_pool_blocks=16)
    import dataclasses
    kv12 = dataclasses.replace(kv, n_kv_heads=12)
    plan = ab.amoeba_plan(shape_from(model_for_kv(kv12), kv12), 2, 3, 0)  # 3 is no multiple of 2
    assert ab.amoeba_plan_merge_factor(plan) == 0
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    rc = ab.amoeba_merge_kv_inplace(plan, buf, [buf], [buf], [buf], buf, check=False)
    assert rc == ab.ERR_INVALID_ARG and "in-place merge" in ab.amoeba_last_error()
    import dataclasses
    tm = dataclasses.replace(kv, layout_src=1)
    plan = ab.amoeba_plan(shape_from(model_for_kv(tm), tm), 1, 2, 0)
    assert ab.amoeba_plan_merge_factor(plan) == 0
    ok = ab.amoeba_plan(shape_from(model_for_kv(kv), kv), 1, 2, 0)
    assert ab.amoeba_plan_merge_factor(ok) == 2
    n = 8 * ab.amoeba_plan_kv_block_bytes(ok, 0)
    pool = torch.zeros(2 * n, dtype=torch.uint8, device="cuda")
    t = torch.zeros((2, 4), dtype=torch.int32, device="cuda")
    l = torch.zeros(2, dtype=torch.int32, device="cuda")
    rc = ab.amoeba_merge_kv_inplace(ok, pool[:n], [None, pool[n // 2:n // 2 + n]], [t, t], [l, l],
                                    torch.zeros((4, 4), dtype=torch.int32, device="cuda"),
                                    check=False)
    assert rc == ab.ERR_INVALID_ARG and "overlap" in ab.amoeba_last_error()


def test_merge_4xTP1_to_TP4_at_7b_block_shape():
    """The paper's scenario at real block geometry: four TP1 instances of the 7B-shaped model
    (32 KV heads, 256 KiB blocks) each serve a quarter of the workload's sequences; target
    rank 1 of TP4 keeps 8 heads in place and receives 8 heads of everybody else's blocks.
    Two layers, so the oracle finishes in seconds."""
    w = wl.WORKLOADS["llama7b"]
    lens_all = wl.seq_lens(w)
    m, k = 4, 1
    per = [lens_all[g::m][:6] for g in range(m)]
    nb_max = max(int(((x.astype(np.int64) + 15) // 16).sum()) for x in per)
    W = int(max(((x.astype(np.int64) + 15) // 16).max() for x in per)) + 3
    cfg, insts = instances(m, k, per, n_heads=w.n_kv_heads, d=w.head_dim, B=16, layers=2,
                           P=int(nb_max * 1.1) + 1, W=W, seed=12)
    check_merge(cfg, insts, m, k, 1)
