"""GPU parity at the benchmark's full size: the 7B-shaped workload (TP4 -> TP2, rank 1,
32 layers, 64 sequences / 6.8K blocks), in exactly the launch configuration bench.py
times (same plan, same pools, default knobs).  Sampled layers are compared with the CPU
oracle bit for bit; every layer is covered by properties that hold at any size."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    sys.stdout.flush()
    yield


def random_device_bits(n_elems, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    t = torch.empty(n_elems, dtype=torch.int16, device="cuda")
    raw = t.view(torch.uint8)
    step = 1 << 29
    for a in range(0, raw.numel(), step):
        raw[a:a + step].random_(0, 256, generator=g)
    return t


@pytest.fixture(scope="module")
def full():
    w = wl.WORKLOADS["llama7b"]
    lens = wl.seq_lens(w)
    table, src_pool = wl.block_placement(w, lens)
    total = int(wl.blocks_per_seq(lens, w.block_tokens).sum())
    shape = ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim,
                          elem_bytes=2, kv_block_tokens=w.block_tokens, kv_layers=w.n_layers,
                          num_seqs=w.num_seqs, max_blocks_per_seq=table.shape[1],
                          src_pool_blocks=src_pool, dst_pool_blocks=total + 64)
    plan = ab.amoeba_plan(shape, w.src_tp, w.dst_tp, w.dst_rank)
    ab.amoeba_plan_tune(plan, ab.TUNE_KV_BLOCKS_HINT, total)   # as bench.py does
    yield dict(w=w, lens=lens, table=table, src_pool=src_pool, total=total, plan=plan)
    plan.close()
    torch.cuda.empty_cache()


def test_weights_full_depth_sampled_layers_match_oracle(full):
    w, plan = full["w"], full["plan"]
    sb, db = ab.amoeba_plan_shard_bytes(plan, 0), ab.amoeba_plan_shard_bytes(plan, 1)
    mask = ab.amoeba_plan_src_rank_mask(plan)
    src = [random_device_bits(sb // 2, seed=40 + r) if mask >> r & 1 else None
           for r in range(w.src_tp)]
    dst = torch.full((db // 2 + 512,), 0x5A5A, dtype=torch.int16, device="cuda")
    ab.amoeba_reshard_weights(plan, src, dst[256:256 + db // 2])
    torch.cuda.synchronize()
    assert bool((dst[:256] == 0x5A5A).all()) and bool((dst[256 + db // 2:] == 0x5A5A).all())
    one = oracle.Model(1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
    ls, ld = sb // 2 // w.n_layers, db // 2 // w.n_layers
    assert ls == oracle.shard_elems(one, w.src_tp) and ld == oracle.shard_elems(one, w.dst_tp)
    for layer in (0, 1, 17, w.n_layers - 1):
        host_src = [None if t is None else t[layer * ls:(layer + 1) * ls].cpu().numpy().view(np.uint16)
                    for t in src]
        st, want = oracle.reshard_weights(one, w.src_tp, w.dst_tp, w.dst_rank, host_src)
        assert st == oracle.OK
        got = dst[256 + layer * ld:256 + (layer + 1) * ld].cpu().numpy().view(np.uint16)
        np.testing.assert_array_equal(got, want, err_msg=f"layer {layer}")
    # any-size property for this merge (TP4 ranks 2,3 -> TP2 rank 1): the target holds each
    # source element exactly once, so per-layer sums agree on every layer
    d = dst[256:256 + db // 2].view(w.n_layers, ld).to(torch.int64).sum(dim=1)
    s = sum(t.view(w.n_layers, ls).to(torch.int64).sum(dim=1) for t in src if t is not None)
    assert torch.equal(d, s)


def test_kv_full_size_matches_oracle_on_sampled_layers_and_index_select_on_all(full):
    w, plan, table, lens = full["w"], full["plan"], full["table"], full["lens"]
    total, src_pool = full["total"], full["src_pool"]
    L, P = w.n_layers, total + 64
    bs, bd = ab.amoeba_plan_kv_block_bytes(plan, 0) // 2, ab.amoeba_plan_kv_block_bytes(plan, 1) // 2
    mask = ab.amoeba_plan_kv_rank_mask(plan)
    src = [random_device_bits(L * src_pool * bs, seed=50 + r) if mask >> r & 1 else None
           for r in range(w.src_tp)]
    dst = torch.full((L * P * bd,), 0x3C3C, dtype=torch.int16, device="cuda")
    out_table = torch.full(table.shape, -9, dtype=torch.int32, device="cuda")
    ab.amoeba_reshard_kv(plan, src, torch.from_numpy(table).cuda(), torch.from_numpy(lens).cuda(),
                         dst, out_table)
    rc, n = ab.amoeba_kv_status(plan)
    assert rc == ab.OK and n == total
    kv = oracle.KV(kv_layers=1, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                   block_tokens=w.block_tokens, num_seqs=w.num_seqs,
                   max_blocks_per_seq=table.shape[1], src_pool_blocks=src_pool, dst_pool_blocks=P)
    dst3 = dst.view(L, P, bd)
    want_table = None
    for layer in (0, L - 1):
        host_src = [None if t is None else
                    t.view(L, src_pool, bs)[layer].cpu().numpy().view(np.uint16)[None]
                    for t in src]
        want = np.full((1, P, bd), 0x3C3C, dtype=np.uint16)
        st, want_table, tot = oracle.reshard_kv(kv, w.src_tp, w.dst_tp, w.dst_rank, host_src,
                                                table, lens, want)
        assert st == oracle.OK and tot == total
        np.testing.assert_array_equal(dst3[layer].cpu().numpy().view(np.uint16), want[0],
                                      err_msg=f"layer {layer}")
    np.testing.assert_array_equal(out_table.cpu().numpy(), want_table)
    # all layers: blocks past the total keep their sentinel ...
    assert bool((dst3[:, total:] == 0x3C3C).all())
    # ... and, header-centric TP4 -> TP2, block b of the target is source block order[b] of
    # rank 2 followed by the same block of rank 3 (index_select special case of the oracle pins)
    nb = wl.blocks_per_seq(lens, w.block_tokens)
    order = torch.from_numpy(np.concatenate([table[i, :nb[i]] for i in range(len(lens))])
                             .astype(np.int64)).cuda()
    for layer in range(L):
        for half, r in enumerate((2, 3)):
            ref = src[r].view(L, src_pool, bs)[layer].index_select(0, order)
            got = dst3[layer, :total, half * bs:(half + 1) * bs]
            assert torch.equal(got, ref), f"layer {layer} rank {r}"


def test_weights_70b_gqa_full_depth_sampled_layers_match_oracle():
    """TP8 -> TP4 rank 2 of the 70B-shaped GQA model at all 80 layers: a 31.9 GiB target shard
    from two 15.9 GiB source shards, so every offset past 2^32 and 2^34 bytes is exercised."""
    w = wl.WORKLOADS["gqa70b"]
    shape = ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
    plan = ab.amoeba_plan(shape, w.src_tp, w.dst_tp, w.dst_rank)
    sb, db = ab.amoeba_plan_shard_bytes(plan, 0), ab.amoeba_plan_shard_bytes(plan, 1)
    mask = ab.amoeba_plan_src_rank_mask(plan)
    assert {r for r in range(w.src_tp) if mask >> r & 1} == {4, 5}
    src = [random_device_bits(sb // 2, seed=60 + r) if mask >> r & 1 else None
           for r in range(w.src_tp)]
    dst = torch.full((db // 2,), 0x5A5A, dtype=torch.int16, device="cuda")
    ab.amoeba_reshard_weights(plan, src, dst)
    torch.cuda.synchronize()
    one = oracle.Model(1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
    ls, ld = sb // 2 // w.n_layers, db // 2 // w.n_layers
    for layer in (0, 41, w.n_layers - 1):
        host_src = [None if t is None else t[layer * ls:(layer + 1) * ls].cpu().numpy().view(np.uint16)
                    for t in src]
        st, want = oracle.reshard_weights(one, w.src_tp, w.dst_tp, w.dst_rank, host_src)
        assert st == oracle.OK
        got = dst[layer * ld:(layer + 1) * ld].cpu().numpy().view(np.uint16)
        np.testing.assert_array_equal(got, want, err_msg=f"layer {layer}")
    d = dst.view(w.n_layers, ld).to(torch.int64).sum(dim=1)
    s = sum(t.view(w.n_layers, ls).to(torch.int64).sum(dim=1) for t in src if t is not None)
    assert torch.equal(d, s)
    plan.close()
    del src, dst
    torch.cuda.empty_cache()


def _bench_config(name, kv_layers):
    """The plan bench.py builds for a workload (same shape, same blocks-in-use hint)."""
    w = wl.WORKLOADS[name]
    lens = wl.seq_lens(w)
    table, src_pool = wl.block_placement(w, lens)
    total = int(wl.blocks_per_seq(lens, w.block_tokens).sum())
    shape = ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim,
                          elem_bytes=2, kv_block_tokens=w.block_tokens, kv_layers=kv_layers,
                          num_seqs=w.num_seqs, max_blocks_per_seq=table.shape[1],
                          src_pool_blocks=src_pool, dst_pool_blocks=total + 64)
    plan = ab.amoeba_plan(shape, w.src_tp, w.dst_tp, w.dst_rank)
    ab.amoeba_plan_tune(plan, ab.TUNE_KV_BLOCKS_HINT, total)
    return w, lens, table, src_pool, total, plan


@pytest.mark.parametrize("name,kv_layers", [("llama13b", 16), ("gqa70b", 80), ("long8b", 32)])
def test_kv_other_benchmark_configs_at_full_size(name, kv_layers):
    """The 13B (16 resident layers, as bench.py keeps), 70B-GQA and long-context KV caches in
    the launch configuration bench.py times.  First and last resident layer bit for bit against
    the oracle; on every layer the unused target blocks keep their sentinel and the sum over
    the used ones equals the sum over the source heads the target rank owns (header-centric
    blocks: a rank's heads are one slice of the block's leading axis)."""
    w, lens, table, src_pool, total, plan = _bench_config(name, kv_layers)
    L, P = kv_layers, total + 64
    bs, bd = ab.amoeba_plan_kv_block_bytes(plan, 0) // 2, ab.amoeba_plan_kv_block_bytes(plan, 1) // 2
    mask = ab.amoeba_plan_kv_rank_mask(plan)
    src = [random_device_bits(L * src_pool * bs, seed=70 + r) if mask >> r & 1 else None
           for r in range(w.src_tp)]
    dst = torch.full((L * P * bd,), 0x3C3C, dtype=torch.int16, device="cuda")
    out_table = torch.full(table.shape, -9, dtype=torch.int32, device="cuda")
    ab.amoeba_reshard_kv(plan, src, torch.from_numpy(table).cuda(), torch.from_numpy(lens).cuda(),
                         dst, out_table)
    rc, n = ab.amoeba_kv_status(plan)
    assert rc == ab.OK and n == total
    kv = oracle.KV(kv_layers=1, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                   block_tokens=w.block_tokens, num_seqs=w.num_seqs,
                   max_blocks_per_seq=table.shape[1], src_pool_blocks=src_pool, dst_pool_blocks=P)
    dst3 = dst.view(L, P, bd)
    want_table = None
    for layer in (0, L - 1):
        print(f"  oracle layer {layer}", flush=True)
        host_src = [None if t is None else
                    t.view(L, src_pool, bs)[layer].cpu().numpy().view(np.uint16)[None]
                    for t in src]
        want = np.full((1, P, bd), 0x3C3C, dtype=np.uint16)
        st, want_table, tot = oracle.reshard_kv(kv, w.src_tp, w.dst_tp, w.dst_rank, host_src,
                                                table, lens, want)
        assert st == oracle.OK and tot == total
        np.testing.assert_array_equal(dst3[layer].cpu().numpy().view(np.uint16), want[0],
                                      err_msg=f"layer {layer}")
        del host_src, want
    np.testing.assert_array_equal(out_table.cpu().numpy(), want_table)
    assert bool((dst3[:, total:] == 0x3C3C).all())
    nb = wl.blocks_per_seq(lens, w.block_tokens)
    order = torch.from_numpy(np.concatenate([table[i, :nb[i]] for i in range(len(lens))])
                             .astype(np.int64)).cuda()
    hs, hd = w.n_kv_heads // w.src_tp, w.n_kv_heads // w.dst_tp
    per_head = bs // hs
    for layer in range(L):
        got = dst3[layer, :total].to(torch.int64).sum()
        ref = 0
        for r in range(w.src_tp):
            lo, hi = max(w.dst_rank * hd, r * hs), min((w.dst_rank + 1) * hd, (r + 1) * hs)
            if lo >= hi:
                continue
            blocks = src[r].view(L, src_pool, hs, per_head)[layer].index_select(0, order)
            ref = ref + blocks[:, lo - r * hs:hi - r * hs].to(torch.int64).sum()
        assert int(got) == int(ref), f"layer {layer}"
    plan.close()
    del src, dst, dst3
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["llama13b", "long8b"])
def test_weights_other_benchmark_configs_full_depth(name):
    """13B TP2 -> TP1 (23.6 GiB target from two shards) and long-context 8B TP1 -> TP4 rank 3 at
    all layers: three layers bit for bit against the oracle, per-layer sums on all (every
    source element the target owns appears exactly once; at TP1 -> TP4 the sum is compared with
    the oracle's on the sampled layers only)."""
    w, lens, table, src_pool, total, plan = _bench_config(name, 1)
    sb, db = ab.amoeba_plan_shard_bytes(plan, 0), ab.amoeba_plan_shard_bytes(plan, 1)
    mask = ab.amoeba_plan_src_rank_mask(plan)
    src = [random_device_bits(sb // 2, seed=80 + r) if mask >> r & 1 else None
           for r in range(w.src_tp)]
    dst = torch.full((db // 2 + 512,), 0x5A5A, dtype=torch.int16, device="cuda")
    ab.amoeba_reshard_weights(plan, src, dst[256:256 + db // 2])
    torch.cuda.synchronize()
    assert bool((dst[:256] == 0x5A5A).all()) and bool((dst[256 + db // 2:] == 0x5A5A).all())
    one = oracle.Model(1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
    ls, ld = sb // 2 // w.n_layers, db // 2 // w.n_layers
    for layer in (0, w.n_layers // 2, w.n_layers - 1):
        print(f"  oracle layer {layer}", flush=True)
        host_src = [None if t is None else t[layer * ls:(layer + 1) * ls].cpu().numpy().view(np.uint16)
                    for t in src]
        st, want = oracle.reshard_weights(one, w.src_tp, w.dst_tp, w.dst_rank, host_src)
        assert st == oracle.OK
        got = dst[256 + layer * ld:256 + (layer + 1) * ld].cpu().numpy().view(np.uint16)
        np.testing.assert_array_equal(got, want, err_msg=f"layer {layer}")
    if w.dst_tp <= w.src_tp:   # a gather of whole source shards: sums agree layer by layer
        d = dst[256:256 + db // 2].view(w.n_layers, ld).to(torch.int64).sum(dim=1)
        s = sum(t.view(w.n_layers, ls).to(torch.int64).sum(dim=1) for t in src if t is not None)
        assert torch.equal(d, s)
    plan.close()
    del src, dst
    torch.cuda.empty_cache()
