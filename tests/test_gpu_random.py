"""GPU parity on seeded random shapes (valid inputs only): weights in the dense, padded and
expert-wise layouts and the KV regroup in all four layout pairs, bit for bit against the oracle,
with guard bands.  The shapes mix vector widths (odd head sizes force 8/4/2/1-byte accesses),
degree pairs that are multiples, divisors and neither, empty sequences and partly filled pools."""
import sys

import numpy as np
import pytest
import torch

import oracle
from gpu_util import gpu_reshard_kv, to_dev
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEGREES = [1, 2, 3, 4, 6, 8, 12, 16]


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    sys.stdout.flush()
    yield


def draw_model(seed):
    rng = np.random.default_rng(5000 + seed)
    k, kp = (int(x) for x in rng.choice(DEGREES, size=2))
    lcm = int(np.lcm(k, kp))
    n_kv = lcm * int(rng.integers(1, 3))
    eb = int(rng.choice([1, 2, 2, 4]))
    d = int(rng.choice([1, 3, 4, 8, 16, 40, 64]))
    m = oracle.Model(n_layers=int(rng.integers(1, 4)), hidden=int(rng.integers(1, 33)) * 8,
                     n_q_heads=n_kv * int(rng.integers(1, 3)), n_kv_heads=n_kv, head_dim=d,
                     ffn_dim=lcm * int(rng.integers(1, 24)), elem_bytes=eb)
    return rng, m, k, kp, int(rng.integers(0, kp))


def run_weights(shape, k, kp, rp, src, want):
    plan = ab.amoeba_plan(shape, k, kp, rp)
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
    np.testing.assert_array_equal(host[guard:guard + n], want.view(np.uint8))
    plan.close()


def base_shape(m, **kw):
    return ab.ModelShape(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_dim,
                         elem_bytes=m.elem_bytes, **kw)


@pytest.mark.parametrize("seed", range(24))
def test_random_weights_dense_padded_expert(seed):
    rng, m, k, kp, rp = draw_model(seed)
    eb = m.elem_bytes
    # dense
    src = [wl.random_bits(oracle.shard_elems(m, k), seed=seed * 17 + r, elem_bytes=eb)
           for r in range(k)]
    st, want = oracle.reshard_weights(m, k, kp, rp, src)
    assert st == oracle.OK
    run_weights(base_shape(m), k, kp, rp, src, want)
    # padded partition-major FFN
    T = int(np.lcm(k, kp))
    page = eb * int(rng.integers(1, 300))
    if T <= ab.MAX_TP:
        sp, dp = [(False, True), (True, True), (True, False)][seed % 3]
        psrc = src
        if sp:
            up = oracle.Pad(T, page, src_padded=False, dst_padded=True)
            psrc = [oracle.reshard_weights_padded(m, up, k, k, r, src)[1] for r in range(k)]
        st, want = oracle.reshard_weights_padded(m, oracle.Pad(T, page, sp, dp), k, kp, rp, psrc)
        assert st == oracle.OK
        run_weights(base_shape(m, w_layout_src=int(sp), w_layout_dst=int(dp), pad_max_tp=T,
                               pad_page_bytes=page), k, kp, rp, psrc, want)
    # expert-wise
    n_exp = int(np.lcm(k, kp)) * int(rng.integers(1, 3))
    sp, dp = [(False, False), (False, True), (True, True), (True, False)][seed % 4]
    flat = oracle.Moe(n_exp)
    esrc = [wl.random_bits(oracle.moe_shard_elems(m, flat, False, k), seed=seed * 23 + r,
                           elem_bytes=eb) for r in range(k)]
    if sp:
        up = oracle.Moe(n_exp, page, False, True)
        esrc = [oracle.reshard_weights_moe(m, up, k, k, r, esrc)[1] for r in range(k)]
    st, want = oracle.reshard_weights_moe(m, oracle.Moe(n_exp, page, sp, dp), k, kp, rp, esrc)
    assert st == oracle.OK
    run_weights(base_shape(m, w_layout_src=int(sp), w_layout_dst=int(dp), n_experts=n_exp,
                           pad_page_bytes=page), k, kp, rp, esrc, want)


@pytest.mark.parametrize("seed", range(24))
def test_random_kv(seed):
    rng = np.random.default_rng(7000 + seed)
    k, kp = (int(x) for x in rng.choice(DEGREES, size=2))
    heads = int(np.lcm(k, kp)) * int(rng.integers(1, 3))
    d = int(rng.choice([1, 3, 4, 8, 16, 32, 64]))
    eb = int(rng.choice([1, 2, 2, 4]))
    B = int(rng.choice([1, 4, 16, 32]))
    S = int(rng.integers(1, 40))
    lens = rng.integers(0, 6 * B + 1, size=S).astype(np.int32)
    lens[rng.integers(0, S)] = 0
    nb = (lens.astype(np.int64) + B - 1) // B
    need = int(nb.sum())
    P = need + int(rng.integers(0, 20))
    W = int(nb.max(initial=0)) + int(rng.integers(0, 3))
    ids = rng.permutation(max(P, 1))[:need]
    table = np.full((S, max(W, 1)), -1, dtype=np.int32)
    p = 0
    for i, n in enumerate(nb):
        table[i, :n] = ids[p:p + n]
        p += int(n)
    lay_s, lay_d = int(rng.integers(0, 2)), int(rng.integers(0, 2))
    layers = int(rng.integers(1, 4))
    kv = oracle.KV(kv_layers=layers, n_kv_heads=heads, head_dim=d, block_tokens=B, num_seqs=S,
                   max_blocks_per_seq=table.shape[1], src_pool_blocks=max(P, 1),
                   dst_pool_blocks=need + int(rng.integers(0, 5)), layout_src=lay_s,
                   layout_dst=lay_d, elem_bytes=eb)
    rp = int(rng.integers(0, kp))
    be_s, be_d = oracle.kv_block_elems(kv, k), oracle.kv_block_elems(kv, kp)
    pools = [wl.random_bits(layers * kv.src_pool_blocks * be_s, seed=seed * 29 + s, elem_bytes=eb)
             .reshape(layers, kv.src_pool_blocks, be_s) for s in range(k)]
    dt = oracle.elem_dtype(eb)
    want = np.full((layers, kv.dst_pool_blocks, be_d), int.from_bytes(b"\xa7" * eb, "little"),
                   dtype=dt)
    st, want_table, total = oracle.reshard_kv(kv, k, kp, rp, pools, table, lens, want)
    assert st == oracle.OK and total == need
    tune = {ab.TUNE_KV_BLOCKS_HINT: need} if seed % 2 else None
    gst, got, got_table, gtotal, intact = gpu_reshard_kv(kv, k, kp, rp, pools, table, lens,
                                                         tune=tune)
    assert gst == ab.OK and gtotal == need and intact
    np.testing.assert_array_equal(got_table, want_table)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("seed", range(16))
def test_random_inplace_merge(seed):
    from test_gpu_merge import check_merge, instances

    rng = np.random.default_rng(9000 + seed)
    m, k = int(rng.choice([2, 3, 4, 8])), int(rng.choice([1, 2]))
    heads = m * k * int(rng.integers(1, 3))
    d = int(rng.choice([1, 4, 8, 32, 64]))
    eb = int(rng.choice([1, 2, 2, 4]))
    B = int(rng.choice([1, 4, 16]))
    S = int(rng.integers(1, 12))
    lens = [rng.integers(0, 5 * B + 1, size=S).tolist() for _ in range(m)]
    worst = max(sum((x + B - 1) // B for x in row) for row in lens)
    P = worst + int(rng.integers(0, 12))
    W = max(1, max((x + B - 1) // B for row in lens for x in row)) + int(rng.integers(0, 2))
    cfg, insts = instances(m, k, lens, n_heads=heads, d=d, B=B, layers=int(rng.integers(1, 4)),
                           P=max(P, 1), W=W, seed=seed + 1, elem_bytes=eb)
    hint = {ab.TUNE_KV_BLOCKS_HINT: m * worst} if seed % 2 else None
    check_merge(cfg, insts, m, k, int(rng.integers(0, k * m)), tune=hint)
