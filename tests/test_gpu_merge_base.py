"""GPU parity of the base solution of Sec. 3.1 (amoeba_merge_kv_base: migration pass, then
de-fragmentation pass, into a second pool) against the oracle: the whole new pool (moved and
untouched bytes alike), the merged table, the status and the block total, bit for bit."""
import dataclasses
import sys

import numpy as np
import pytest
import torch

import oracle
from gpu_util import model_for_kv, shape_from, to_dev
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl
from test_gpu_merge import instances

pytestmark = pytest.mark.gpu

HM, TM = ab.KV_HEAD_MAJOR, ab.KV_TOKEN_MAJOR


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    sys.stdout.flush()
    yield


def check_base(cfg, insts, m, k, rp, lay=(TM, TM), slack=3, expect=oracle.OK, tune=None, bound=0,
               pool_blocks=None, local_bound=0):
    s = rp // m
    tabs, lens = [i["table"] for i in insts], [i["lens"] for i in insts]
    pools = [insts[g2]["pools"][s] for g2 in range(m)]
    total = sum(int(((np.maximum(x, 0).astype(np.int64) + cfg.block_tokens - 1)
                     // cfg.block_tokens).sum()) for x in lens)
    cfg = dataclasses.replace(cfg, layout_src=lay[0], layout_dst=lay[1],
                              dst_pool_blocks=total + slack if pool_blocks is None else pool_blocks)
    be = oracle.kv_block_elems(cfg, k * m)
    dt = oracle.elem_dtype(cfg.elem_bytes)
    sent = int.from_bytes(b"\xa7" * cfg.elem_bytes, "little")
    want = np.full((cfg.kv_layers, cfg.dst_pool_blocks, be), sent, dtype=dt)
    ost, want_table, mig, dfr = oracle.merge_kv_base(cfg, k, m, rp, pools, tabs, lens, want)
    assert ost == expect

    shape = shape_from(model_for_kv(cfg), cfg)
    shape.kv_blocks_bound = bound
    plan = ab.amoeba_plan(shape, k, k * m, rp)
    for knob, val in (tune or {}).items():
        ab.amoeba_plan_tune(plan, knob, val)
    n_bytes = want.nbytes
    guard = 4096
    buf = torch.full((n_bytes + 2 * guard,), 0xA7, dtype=torch.uint8, device="cuda")
    out_table = torch.full((m * cfg.num_seqs, cfg.max_blocks_per_seq), -9, dtype=torch.int32,
                           device="cuda")
    ab.amoeba_merge_kv_base(plan, [to_dev(a) for a in pools],
                            [torch.from_numpy(t).cuda() for t in tabs],
                            [torch.from_numpy(x).cuda() for x in lens],
                            buf[guard:guard + n_bytes], out_table, local_bound)
    st, n = ab.amoeba_kv_status(plan)
    code = {oracle.OK: ab.OK, oracle.ERR_OVERFLOW: ab.ERR_OVERFLOW,
            oracle.ERR_BLOCK_ID: ab.ERR_BLOCK_ID}[ost]
    assert st == code
    assert n == (0 if ost == oracle.ERR_OVERFLOW else total)
    host = buf.cpu().numpy()
    assert (host[:guard] == 0xA7).all() and (host[guard + n_bytes:] == 0xA7).all()
    np.testing.assert_array_equal(out_table.cpu().numpy(), want_table)
    np.testing.assert_array_equal(host[guard:guard + n_bytes].view(dt).reshape(want.shape), want)
    plan.close()


LENS4 = [[13, 1, 8, 0, 40], [5, 22, 3, 9, 0], [16, 2, 7, 7, 1], [1, 1, 30, 4, 12]]


@pytest.mark.parametrize("lay", [(TM, TM), (HM, HM), (TM, HM), (HM, TM)])
@pytest.mark.parametrize("m,k,n_heads", [(4, 1, 8), (2, 1, 8), (2, 2, 8), (3, 2, 12), (2, 4, 16)])
def test_base_merge_small_every_target_rank(m, k, n_heads, lay):
    cfg, insts = instances(m, k, LENS4[:m], n_heads=n_heads, d=8, B=4, layers=3, P=40, W=14,
                           seed=m * 7 + k)
    for rp in range(k * m):
        check_base(cfg, insts, m, k, rp, lay=lay)


@pytest.mark.parametrize("elem_bytes,d", [(2, 64), (1, 16), (4, 4), (2, 4), (2, 2), (2, 1), (1, 1)])
def test_base_merge_every_vector_width_and_launch_shape(elem_bytes, d):
    """d = 64 at 16 bits: 16 KiB new blocks, several tiles each; small d falls back to
    8/4/2/1-byte accesses.  Launch shapes: one or four wavefronts per workgroup, 1-4 vectors per
    lane, grids bounded by a bound that is too small (workgroups stride), exact, or absent."""
    cfg, insts = instances(2, 1, [[33, 7, 100], [64, 1, 18]], n_heads=4, d=d, B=16, layers=2,
                           P=16, W=9, seed=d, elem_bytes=elem_bytes)
    for rp in range(2):
        check_base(cfg, insts, 2, 1, rp)
        check_base(cfg, insts, 2, 1, rp, lay=(TM, HM))
    check_base(cfg, insts, 2, 1, 1, tune={ab.TUNE_KV_GRID: 3, ab.TUNE_NONTEMPORAL: 2})
    for threads, unroll, bound in [(64, 1, 1), (256, 2, 1), (64, 4, 17), (256, 1, 17), (0, 0, 0),
                                   (0, 0, 17), (256, 4, 0), (0, 0, 10000)]:
        check_base(cfg, insts, 2, 1, 0, bound=bound,
                   tune={ab.TUNE_KV_THREADS: threads, ab.TUNE_KV_UNROLL: unroll})
    # per-pass grids: exact local bound (10 blocks of 17), too small, larger than the whole
    for local in (10, 1, 40):
        check_base(cfg, insts, 2, 1, 0, bound=17, local_bound=local)
    check_base(cfg, insts, 2, 1, 1, bound=0, local_bound=7)    # a local bound alone changes nothing


def test_base_merge_degenerate_and_error_cases():
    cfg, insts = instances(2, 1, [[0, 0], [0, 0]], n_heads=4, d=8, B=4, layers=1, P=8, W=4, seed=1)
    check_base(cfg, insts, 2, 1, 0)                        # nothing to move
    check_base(cfg, insts, 2, 1, 0, slack=0)               # and a new pool of zero blocks
    cfg, insts = instances(2, 1, [[9, 4], [0, 0]], n_heads=4, d=8, B=4, layers=2, P=8, W=4, seed=4)
    check_base(cfg, insts, 2, 1, 0)                        # only local requests: pass 1 is empty
    check_base(cfg, insts, 2, 1, 1)                        # only remote requests: pass 2 is empty
    cfg, insts = instances(2, 1, [[9, 4], [5, 8]], n_heads=4, d=8, B=4, layers=2, P=8, W=4, seed=2)
    check_base(cfg, insts, 2, 1, 0, slack=0)               # exact fit
    check_base(cfg, insts, 2, 1, 0, pool_blocks=3 + 1 + 2 + 2 - 1, expect=oracle.ERR_OVERFLOW)
    insts[1]["lens"][0] = -3
    check_base(cfg, insts, 2, 1, 0, expect=oracle.ERR_OVERFLOW)
    insts[1]["lens"][0] = 5
    check_base(cfg, insts, 2, 1, 0)                        # the status resets between calls
    insts[0]["lens"][1] = 4 * 4 + 1                        # needs 5 blocks, the row holds 4
    check_base(cfg, insts, 2, 1, 1, expect=oracle.ERR_OVERFLOW)
    insts[0]["lens"][1] = 4
    insts[1]["table"][1, 0] = 8                            # one past the pool
    check_base(cfg, insts, 2, 1, 0, expect=oracle.ERR_BLOCK_ID)
    insts[0]["table"][0, 1] = -2                           # a bad id in the local table
    check_base(cfg, insts, 2, 1, 0, expect=oracle.ERR_BLOCK_ID)


def test_base_merge_rejects_plans_that_are_not_a_merge():
    kv = oracle.KV(kv_layers=1, n_kv_heads=12, head_dim=8, block_tokens=4, num_seqs=2,
                   max_blocks_per_seq=4, src_pool_blocks=8, dst_pool_blocks=16)
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    for k, kp in [(2, 3), (2, 2), (4, 2)]:
        plan = ab.amoeba_plan(shape_from(model_for_kv(kv), kv), k, kp, 0)
        rc = ab.amoeba_merge_kv_base(plan, [buf] * 4, [buf] * 4, [buf] * 4, buf, buf, check=False)
        assert rc == ab.ERR_INVALID_ARG and "merge of instances" in ab.amoeba_last_error()
        plan.close()
    plan = ab.amoeba_plan(shape_from(model_for_kv(kv), kv), 1, 2, 0)
    n = 8 * ab.amoeba_plan_kv_block_bytes(plan, 0)
    pool = torch.zeros(3 * n, dtype=torch.uint8, device="cuda")
    t = torch.zeros((2, 4), dtype=torch.int32, device="cuda")
    l = torch.zeros(2, dtype=torch.int32, device="cuda")
    rc = ab.amoeba_merge_kv_base(plan, [pool[:n], pool[n:2 * n]], [t, t], [l, l],
                                 pool[n + n // 2:], torch.zeros((4, 4), dtype=torch.int32,
                                                                device="cuda"), check=False)
    assert rc == ab.ERR_INVALID_ARG and "overlap" in ab.amoeba_last_error()
    plan.close()


@pytest.mark.parametrize("lay", [(TM, TM), (HM, HM)])
def test_base_merge_4xTP1_to_TP4_at_7b_block_shape(lay):
    """The paper's scenario at real block geometry: four TP1 instances of the 7B-shaped model
    (32 KV heads, 256 KiB blocks), target rank 1 of TP4, two layers."""
    w = wl.WORKLOADS["llama7b"]
    lens_all = wl.seq_lens(w)
    m, k = 4, 1
    per = [lens_all[g::m][:6] for g in range(m)]
    nb_max = max(int(((x.astype(np.int64) + 15) // 16).sum()) for x in per)
    W = int(max(((x.astype(np.int64) + 15) // 16).max() for x in per)) + 3
    cfg, insts = instances(m, k, per, n_heads=w.n_kv_heads, d=w.head_dim, B=16, layers=2,
                           P=int(nb_max * 1.1) + 1, W=W, seed=12)
    total = sum(int(((x.astype(np.int64) + 15) // 16).sum()) for x in per)
    local = int(((per[1].astype(np.int64) + 15) // 16).sum())
    check_base(cfg, insts, m, k, 1, lay=lay, bound=total, local_bound=local)


@pytest.mark.parametrize("seed", range(12))
def test_base_merge_random_shapes(seed):
    rng = np.random.default_rng(4000 + seed)
    m = int(rng.choice([2, 2, 3, 4]))
    k = int(rng.choice([1, 1, 2]))
    heads = m * k * int(rng.integers(1, 3))
    d = int(rng.choice([1, 4, 8, 32, 64]))
    eb = int(rng.choice([1, 2, 2, 4]))
    B = int(rng.choice([1, 4, 16]))
    S = int(rng.integers(1, 12))
    lens = [rng.integers(0, 5 * B + 1, size=S).tolist() for _ in range(m)]
    worst = max(sum((x + B - 1) // B for x in row) for row in lens)
    W = max(1, max((x + B - 1) // B for row in lens for x in row)) + int(rng.integers(0, 2))
    cfg, insts = instances(m, k, lens, n_heads=heads, d=d, B=B, layers=int(rng.integers(1, 4)),
                           P=max(worst + int(rng.integers(0, 12)), 1), W=W, seed=seed + 1,
                           elem_bytes=eb)
    lay = (int(rng.integers(0, 2)), int(rng.integers(0, 2)))
    total = sum(sum((x + B - 1) // B for x in row) for row in lens)
    check_base(cfg, insts, m, k, int(rng.integers(0, k * m)), lay=lay,
               slack=int(rng.integers(0, 5)), bound=total if seed % 2 else 0,
               local_bound=int(rng.integers(0, total + 2)) if seed % 3 else 0)
