"""GPU parity at the benchmark's full sizes, in the launch configurations bench.py times
(same shapes, same pools, the blocks-in-use bound in the shape, default launch choices).

Every layer of every case is compared element by element on the device against a reference
built here with torch slicing only (narrow / cat for the weights, index_select / permute for
the cache: the special cases the oracle is pinned to on the CPU, restated for device
tensors), and sampled layers are compared bit for bit with the CPU oracle itself."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl

pytestmark = pytest.mark.gpu

HM, TM = ab.KV_HEAD_MAJOR, ab.KV_TOKEN_MAJOR
LAYOUTS = {"hm": HM, "tm": TM}


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    sys.stdout.flush()
    yield
    torch.cuda.empty_cache()


def random_device_bits(n_elems, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    t = torch.empty(n_elems, dtype=torch.int16, device="cuda")
    raw = t.view(torch.uint8)
    step = 1 << 29
    for a in range(0, raw.numel(), step):
        raw[a:a + step].random_(0, 256, generator=g)
    return t


# ------------------------------------------------------------------ weights
def unpack_layer(flat, w, tp):
    """Views of one layer of a rank's packed shard (the storage convention: q, k, v, o, gate,
    up, down, row-major [out, in], back to back)."""
    H, d = w.hidden, w.head_dim
    shapes = [("q", (w.n_q_heads * d // tp, H)), ("k", (w.n_kv_heads * d // tp, H)),
              ("v", (w.n_kv_heads * d // tp, H)), ("o", (H, w.n_q_heads * d // tp)),
              ("g", (w.ffn_dim // tp, H)), ("u", (w.ffn_dim // tp, H)),
              ("d", (H, w.ffn_dim // tp))]
    out, p = {}, 0
    for name, (r, c) in shapes:
        out[name] = flat[p:p + r * c].view(r, c)
        p += r * c
    assert p == flat.numel()
    return out


def expected_tensor(name, src_views, k, kp, rp):
    """The target rank's slice of one tensor: its index range along the cut axis (stored rows
    for q, k, v, gate, up; stored columns for o, down), gathered from the ranks that own it."""
    axis = 1 if name in ("o", "d") else 0
    per_src = next(v for v in src_views if v is not None)[name].shape[axis]
    per_dst = per_src * k // kp
    lo, hi = rp * per_dst, (rp + 1) * per_dst
    pieces = []
    for r in range(k):
        a, b = max(lo, r * per_src), min(hi, (r + 1) * per_src)
        if a < b:
            pieces.append(src_views[r][name].narrow(axis, a - r * per_src, b - a))
    return pieces[0] if len(pieces) == 1 else torch.cat(pieces, dim=axis)


def check_weights_full_depth(w, n_layers, oracle_layers, seed):
    shape = ab.ModelShape(n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
    plan = ab.amoeba_plan(shape, w.src_tp, w.dst_tp, w.dst_rank)
    sb, db = ab.amoeba_plan_shard_bytes(plan, 0), ab.amoeba_plan_shard_bytes(plan, 1)
    mask = ab.amoeba_plan_src_rank_mask(plan)
    src = [random_device_bits(sb // 2, seed=seed + r) if mask >> r & 1 else None
           for r in range(w.src_tp)]
    dst = torch.full((db // 2 + 512,), 0x5A5A, dtype=torch.int16, device="cuda")
    ab.amoeba_reshard_weights(plan, src, dst[256:256 + db // 2])
    torch.cuda.synchronize()
    assert bool((dst[:256] == 0x5A5A).all()) and bool((dst[256 + db // 2:] == 0x5A5A).all())
    one = oracle.Model(1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
    ls, ld = sb // 2 // n_layers, db // 2 // n_layers
    assert ls == oracle.shard_elems(one, w.src_tp) and ld == oracle.shard_elems(one, w.dst_tp)
    body = dst[256:256 + db // 2]
    for layer in range(n_layers):        # every layer, every tensor, element by element
        views = [None if t is None else unpack_layer(t[layer * ls:(layer + 1) * ls], w, w.src_tp)
                 for t in src]
        got = unpack_layer(body[layer * ld:(layer + 1) * ld], w, w.dst_tp)
        for name in ("q", "k", "v", "o", "g", "u", "d"):
            want = expected_tensor(name, views, w.src_tp, w.dst_tp, w.dst_rank)
            assert torch.equal(got[name], want), f"layer {layer} tensor {name}"
    for layer in oracle_layers:
        print(f"  oracle layer {layer}", flush=True)
        host_src = [None if t is None else t[layer * ls:(layer + 1) * ls].cpu().numpy().view(np.uint16)
                    for t in src]
        st, want = oracle.reshard_weights(one, w.src_tp, w.dst_tp, w.dst_rank, host_src)
        assert st == oracle.OK
        got = body[layer * ld:(layer + 1) * ld].cpu().numpy().view(np.uint16)
        np.testing.assert_array_equal(got, want, err_msg=f"layer {layer}")
    plan.close()


@pytest.mark.parametrize("name", ["llama7b", "llama13b", "gqa70b", "long8b"])
def test_weights_full_depth_every_layer(name):
    """All layers of each benchmark model in one launch (13B: a 23.6 GiB target from two
    shards; 70B-GQA: 31.9 GiB from two 15.9 GiB shards, offsets past 2^34 bytes)."""
    w = wl.WORKLOADS[name]
    check_weights_full_depth(w, w.n_layers, (0, w.n_layers // 2, w.n_layers - 1), seed=40 + w.index)


def test_weights_target_shard_beyond_one_grid_dimension():
    """A 70B-shaped TP2 -> TP1 merge of 41 layers: the 65 GiB target has more 1 KiB tiles than
    one grid dimension holds at 64 lanes, so the launch is clamped and workgroups stride."""
    w = wl.WORKLOADS["gqa70b"].scaled(src_tp=2, dst_tp=1, dst_rank=0)
    shape = ab.ModelShape(41, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
    plan = ab.amoeba_plan(shape, 2, 1, 0)
    gx, _, lanes, items = ab.amoeba_plan_launch_shape(plan, ab.KERNEL_WEIGHTS, 16)
    assert gx < items and gx * lanes <= 2 ** 32 - 1
    plan.close()
    check_weights_full_depth(w, 41, (0, 40), seed=90)


# ------------------------------------------------------------------ KV cache
def logical_blocks(pool_layer, layout, heads, B, d):
    """[blocks, head, K/V, token, d] view of one layer of a pool, whatever its storage order."""
    n = pool_layer.shape[0]
    if layout == HM:                                  # stored [head][K/V][token][d]
        return pool_layer.view(n, heads, 2, B, d)
    return pool_layer.view(n, 2, B, heads, d).permute(0, 3, 1, 2, 4)   # [K/V][token][head][d]


def bench_setup(name, kv_layers, layout=("hm", "hm"), bound=True):
    """The plan and the pools bench.py builds for a workload."""
    w = wl.WORKLOADS[name]
    lens = wl.seq_lens(w)
    table, src_pool = wl.block_placement(w, lens)
    total = int(wl.blocks_per_seq(lens, w.block_tokens).sum())
    lay_s, lay_d = LAYOUTS[layout[0]], LAYOUTS[layout[1]]
    shape = ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim,
                          elem_bytes=2, kv_block_tokens=w.block_tokens, kv_layout_src=lay_s,
                          kv_layout_dst=lay_d, kv_layers=kv_layers, num_seqs=w.num_seqs,
                          max_blocks_per_seq=table.shape[1], src_pool_blocks=src_pool,
                          dst_pool_blocks=total + 64, kv_blocks_bound=total if bound else 0)
    plan = ab.amoeba_plan(shape, w.src_tp, w.dst_tp, w.dst_rank)
    return w, lens, table, src_pool, total, plan, lay_s, lay_d


def check_kv_call(w, lens, table, src_pool, total, plan, lay_s, lay_d, L, src, dst, oracle_layers):
    """One amoeba_reshard_kv call over L resident layers, checked on every layer."""
    P = total + 64
    B, d = w.block_tokens, w.head_dim
    hs, hd = w.n_kv_heads // w.src_tp, w.n_kv_heads // w.dst_tp
    bs, bd = hs * 2 * B * d, hd * 2 * B * d
    assert ab.amoeba_plan_kv_block_bytes(plan, 0) == 2 * bs
    assert ab.amoeba_plan_kv_block_bytes(plan, 1) == 2 * bd
    dst.fill_(0x3C3C)
    out_table = torch.full(table.shape, -9, dtype=torch.int32, device="cuda")
    ab.amoeba_reshard_kv(plan, src, torch.from_numpy(table).cuda(), torch.from_numpy(lens).cuda(),
                         dst, out_table)
    rc, n = ab.amoeba_kv_status(plan)
    assert rc == ab.OK and n == total
    dst3 = dst[:L * P * bd].view(L, P, bd)
    # the new table: compact ids in sequence order, -1 behind them
    nb = wl.blocks_per_seq(lens, w.block_tokens)
    want_table = np.full(table.shape, -1, dtype=np.int32)
    base = 0
    for i, c in enumerate(nb):
        want_table[i, :c] = np.arange(base, base + c)
        base += int(c)
    np.testing.assert_array_equal(out_table.cpu().numpy(), want_table)
    # unused target blocks keep their sentinel on every layer
    assert bool((dst3[:, total:] == 0x3C3C).all())
    # every layer: target block b holds, for each head the rank owns, that head of source
    # block order[b] on the rank that owns it
    order = torch.from_numpy(np.concatenate([table[i, :nb[i]] for i in range(len(lens))])
                             .astype(np.int64)).cuda()
    h0 = w.dst_rank * hd
    for layer in range(L):
        got = logical_blocks(dst3[layer, :total], lay_d, hd, B, d)
        for r in range(w.src_tp):
            lo, hi = max(h0, r * hs), min(h0 + hd, (r + 1) * hs)
            if lo >= hi:
                continue
            pool = src[r][:L * src_pool * bs].view(L, src_pool, bs)[layer]
            ref = logical_blocks(pool, lay_s, hs, B, d)[:, lo - r * hs:hi - r * hs]
            ref = ref.index_select(0, order)
            assert torch.equal(got[:, lo - h0:hi - h0], ref), f"layer {layer} source rank {r}"
            del ref
    kv = oracle.KV(kv_layers=1, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                   block_tokens=w.block_tokens, num_seqs=w.num_seqs,
                   max_blocks_per_seq=table.shape[1], src_pool_blocks=src_pool, dst_pool_blocks=P,
                   layout_src=lay_s, layout_dst=lay_d)
    for layer in oracle_layers:
        print(f"  oracle layer {layer}", flush=True)
        host_src = [None if t is None else
                    t[:L * src_pool * bs].view(L, src_pool, bs)[layer].cpu().numpy().view(np.uint16)[None]
                    for t in src]
        want = np.full((1, P, bd), 0x3C3C, dtype=np.uint16)
        st, otable, tot = oracle.reshard_kv(kv, w.src_tp, w.dst_tp, w.dst_rank, host_src, table,
                                            lens, want)
        assert st == oracle.OK and tot == total
        np.testing.assert_array_equal(otable, want_table)
        np.testing.assert_array_equal(dst3[layer].cpu().numpy().view(np.uint16), want[0],
                                      err_msg=f"layer {layer}")
        del host_src, want


def run_kv_case(name, kv_layers, layout=("hm", "hm"), bound=True, oracle_layers=None):
    w, lens, table, src_pool, total, plan, lay_s, lay_d = bench_setup(name, kv_layers, layout, bound)
    L, P = kv_layers, total + 64
    bs = ab.amoeba_plan_kv_block_bytes(plan, 0) // 2
    bd = ab.amoeba_plan_kv_block_bytes(plan, 1) // 2
    mask = ab.amoeba_plan_kv_rank_mask(plan)
    src = [random_device_bits(L * src_pool * bs, seed=50 + 7 * w.index + r) if mask >> r & 1
           else None for r in range(w.src_tp)]
    dst = torch.empty(L * P * bd, dtype=torch.int16, device="cuda")
    if oracle_layers is None:
        oracle_layers = (0, L - 1)
    check_kv_call(w, lens, table, src_pool, total, plan, lay_s, lay_d, L, src, dst, oracle_layers)
    plan.close()
    return w, lens, table, src_pool, total, src, dst


@pytest.mark.parametrize("name,kv_layers", [("llama7b", 32), ("gqa70b", 80), ("long8b", 32)])
def test_kv_full_size_header_centric(name, kv_layers):
    """The 7B, 70B-GQA and long-context caches whole, as bench.py times them."""
    run_kv_case(name, kv_layers)


def test_kv_13b_in_three_calls_over_sixteen_resident_layers():
    """The 13B cache does not fit beside its target (40 layers, about 494 GB), so bench.py
    keeps 16 layers resident and covers the model with calls of 16, 16 and 8 layers over
    those pools; the 8-layer call is a plan of its own.  Both plans are checked on every
    layer they touch."""
    w, lens, table, src_pool, total, src, dst = run_kv_case("llama13b", 16)
    _, _, _, _, _, rest, lay_s, lay_d = bench_setup("llama13b", 8)
    check_kv_call(w, lens, table, src_pool, total, rest, lay_s, lay_d, 8, src, dst, (7,))
    rest.close()


@pytest.mark.parametrize("name,kv_layers", [("llama7b", 32), ("gqa70b", 80)])
@pytest.mark.parametrize("layout", [("tm", "tm"), ("tm", "hm"), ("hm", "tm")])
def test_kv_full_size_other_layout_pairs(name, kv_layers, layout):
    """Token-first on either side at full size (the layout pairs the measurement names)."""
    run_kv_case(name, kv_layers, layout=layout, oracle_layers=(kv_layers - 1,))


@pytest.mark.parametrize("name,kv_layers", [("llama7b", 32), ("long8b", 32)])
def test_kv_full_size_without_the_blocks_bound(name, kv_layers):
    """No bound on the blocks in use: the grid covers the pool's capacity with four-wavefront
    workgroups."""
    run_kv_case(name, kv_layers, bound=False, oracle_layers=(kv_layers // 2,))
