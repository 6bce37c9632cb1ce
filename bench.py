#!/usr/bin/env python3
"""Benchmark of the TP reshard hot path on one MI355X.

One *step* is one pass of the whole hot path for one target rank: plan lookup is
done once outside (it is host-only), then `amoeba_reshard_weights` over all
layers and `amoeba_reshard_kv` (scan + table rewrite + block regroup) over the
whole paged cache, with every input already resident in HBM.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama7b]

prints ONE JSON line.  `value` is read+write GB/s over the algorithmic bytes
(2 x bytes of the target shard and of the target KV blocks in use).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0  # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all",
                    help="all (default): the four 7B-and-larger configurations in one run, the "
                         "headline being the largest (llama13b); or one of tiny, llama7b, "
                         "llama13b, gqa70b, long8b, qwen3moe")
    ap.add_argument("--placement", default="workload", choices=["workload", "sorted"],
                    help="sorted: diagnostic, the workload's source block ids in ascending order")
    ap.add_argument("--no-bound", action="store_true",
                    help="reshard mode: leave amoeba_model_shape.kv_blocks_bound at 0 in the "
                         "timed plan (the run reports both rates either way)")
    ap.add_argument("--layout", default="hm-hm", choices=["hm-hm", "tm-tm", "tm-hm", "hm-tm"])
    ap.add_argument("--kv-layers", type=int, default=0,
                    help="KV layers resident per call (0 = all that fit the workload definition)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="reshard mode: also capture one step in a HIP graph and time its replays "
                         "(what a launch-bound configuration such as `tiny` gains from it)")
    ap.add_argument("--head-dim", type=int, default=0,
                    help="override the workload's head_dim (with --kv-heads: other head geometries "
                         "on the same sequence table, e.g. 64-byte head vectors)")
    ap.add_argument("--kv-heads", type=int, default=0, help="override n_kv_heads = n_q_heads")
    ap.add_argument("--tune", default="", help="knob=value,... (AMOEBA_TUNE_* names, lower case)")
    ap.add_argument("--mode", default="reshard", choices=["reshard", "merge-inplace", "merge-naive", "merge-base", "weights-padded", "overlap"],
                    help="reshard: the TP k -> k' hot path (default, the headline metric); "
                         "merge-inplace: m x TP1 instances -> TP m, KV cache only, in place; "
                         "merge-base (alias merge-naive): the same scenario the paper's base "
                         "way (token-first blocks, migration pass + de-fragmentation pass into "
                         "a second pool); "
                         "weights-padded: TP1 <-> TP4 weight transformation with the padded "
                         "FFN layout against the dense layout (the paper's partial swap); "
                         "overlap: n layers per step resharded on a side stream while a synthetic "
                         "inference step runs on the main stream")
    ap.add_argument("--instances", type=int, default=4, help="m for --mode merge-inplace")
    return ap.parse_args()


HEADLINE = "llama13b"                                     # the largest single-GPU configuration
DEFAULT_SET = ["llama7b", "gqa70b", "long8b", "llama13b"]  # every 7B-and-larger configuration


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share of the reshard on one GPU; "
              "--gpus must be 1 (no collectives or multi-GPU sharding are part of it)",
              file=sys.stderr)
        sys.exit(2)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.mode == "merge-inplace":
        return merge_inplace(args)
    if args.mode in ("merge-naive", "merge-base"):
        return merge_naive(args)
    if args.mode == "weights-padded":
        return weights_padded(args)
    if args.mode == "overlap":
        return overlap(args)

    if args.workload != "all":
        warm_up_device()
        out = reshard(args, args.workload, cpu_budget_s=0 if args.no_cpu_baseline else 12.0)
        print(json.dumps(out), flush=True)
        return
    # Default: every 7B-and-larger configuration in one run.  The headline fields are those of
    # the largest one; `configs` carries the others, each timed the same way (W warm-ups, K
    # timed steps) on its own pools, which are freed before the next one is built.
    rows = []
    head = None
    warm_up_device()
    for name in DEFAULT_SET:
        is_head = name == HEADLINE
        budget = 0 if args.no_cpu_baseline else (15.0 if is_head else 4.0)
        out = reshard(args, name, cpu_budget_s=budget)
        print(f"bench.py: {name}: {out['value']} GB/s, {out['ms_per_step']} ms/step",
              file=sys.stderr, flush=True)
        if is_head:
            head = out
        rows.append(summary_row(name, out))
    head["configs"] = rows
    print(json.dumps(head), flush=True)


def warm_up_device():
    """About a third of a second of streaming copies before the first configuration: the first
    kernels after process start run below the sustained rate (clocks and power state ramp up),
    which would otherwise be charged to whichever configuration comes first."""
    import torch

    from paper_2509_19729_amd import binding as ab
    a = torch.empty(1 << 28, dtype=torch.int32, device="cuda")
    b = torch.empty_like(a)
    a.zero_()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.3:
        for _ in range(20):
            ab.amoeba_copy_baseline(b, a, a.numel() * 4, 64, 1, 0, 1)
        torch.cuda.synchronize()
    del a, b
    torch.cuda.empty_cache()


def summary_row(name, out):
    c, r = out["config"], out["roofline"]
    row = {"workload": name, "gbps": out["value"], "pct_of_hbm_peak": out["pct_of_hbm_peak"],
           "ms_per_tp_transform": out["ms_per_step"], "alg_bytes": c["weights_alg_bytes"] + c["kv_alg_bytes"],
           "weights_ms": c["weights_ms"], "weights_gbps": c["weights_gbps"], "kv_ms": c["kv_ms"],
           "kv_gbps": c["kv_gbps"], "kv_gbps_without_bound": c["kv_gbps_without_bound"],
           "dominant_kernel": r["kernel"], "frac": r["frac"], "avg_launch_ms": r["avg_launch_ms"],
           "plain_copy_gbps": c["plain_copy_gbps"], "tune": c["tune"]}
    if "cpu_baseline" in out:
        row["oracle_gbps"] = out["cpu_baseline"]["value"]
        row["oracle_sample"] = out["cpu_baseline"]["sample"]
    return row


def kernel_sources_digest():
    """SHA-256 over the library's sources: a profile summary under profiles/ records the
    digest of the build it was taken on, and its traffic figure is only quoted for that build."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2509_19729_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def reshard(args, workload, cpu_budget_s):
    """One configuration: W warm-up steps, K timed steps, the side measurements (outside the
    timed region), the oracle sample.  Returns the JSON object."""
    import numpy as np
    import torch

    from paper_2509_19729_amd import binding as ab
    from paper_2509_19729_amd import workloads as wl

    w = wl.WORKLOADS[workload]
    if args.head_dim or args.kv_heads:
        heads = args.kv_heads or w.n_kv_heads
        w = w.scaled(head_dim=args.head_dim or w.head_dim, n_kv_heads=heads, n_q_heads=heads,
                     name=f"{w.name}-d{args.head_dim or w.head_dim}-h{heads}")
    lay = {"hm": ab.KV_HEAD_MAJOR, "tm": ab.KV_TOKEN_MAJOR}
    lay_s, lay_d = (lay[x] for x in args.layout.split("-"))

    lens = wl.seq_lens(w)
    table, src_pool_blocks = wl.block_placement(w, lens)
    if args.placement == "sorted":
        # diagnostic: the same set of source ids, ascending along the new block order, so that
        # the reads sweep the source pools monotonically like the writes sweep the target
        used = table >= 0
        table = table.copy()
        table[used] = np.sort(table[used])
    total_blocks = int(wl.blocks_per_seq(lens, w.block_tokens).sum())
    dst_pool_blocks = total_blocks + 64
    kv_layers = args.kv_layers or w.n_layers
    if w.name == "llama13b" and not args.kv_layers:
        kv_layers = 16  # the full 40-layer cache (src + dst, about 494 GB) exceeds the 288 GB of HBM
    knobs = {n[len("TUNE_"):].lower(): getattr(ab, n) for n in dir(ab) if n.startswith("TUNE_")}

    def make_plan(layers, bound):
        # the scheduler that owns the block tables knows how many blocks are in use and says so
        # in the shape; the library only sees device-side lengths and would otherwise size its
        # grid by the pool's capacity
        shape = ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim,
                              w.ffn_dim, elem_bytes=w.elem_bytes, kv_block_tokens=w.block_tokens,
                              kv_layout_src=lay_s, kv_layout_dst=lay_d, kv_layers=layers,
                              num_seqs=w.num_seqs, max_blocks_per_seq=table.shape[1],
                              src_pool_blocks=src_pool_blocks, dst_pool_blocks=dst_pool_blocks,
                              n_experts=w.n_experts, kv_blocks_bound=bound)
        p = ab.amoeba_plan(shape, w.src_tp, w.dst_tp, w.dst_rank)
        for kv in filter(None, args.tune.split(",")):
            name, val = kv.split("=")
            ab.amoeba_plan_tune(p, knobs[name], int(val))
        return p

    bound = 0 if args.no_bound else total_blocks
    plan = make_plan(kv_layers, bound)

    # ---- synthetic state, generated on the device (values ~ N(0, 0.02), 16-bit) ----
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0xA30EBA00 + w.index)
    fdt = torch.float16 if w.dtype == "fp16" else torch.bfloat16

    def payload(n_elems):
        t = torch.empty(n_elems, dtype=fdt, device="cuda")
        step = 1 << 28
        for a in range(0, n_elems, step):
            t[a:a + step].normal_(0.0, 0.02, generator=gen)
        return t

    src_bytes, dst_bytes = ab.amoeba_plan_shard_bytes(plan, 0), ab.amoeba_plan_shard_bytes(plan, 1)
    wmask, kmask = ab.amoeba_plan_src_rank_mask(plan), ab.amoeba_plan_kv_rank_mask(plan)
    w_src = [payload(src_bytes // 2) if wmask >> r & 1 else None for r in range(w.src_tp)]
    w_dst = torch.empty(dst_bytes // 2, dtype=fdt, device="cuda")
    bb_s, bb_d = ab.amoeba_plan_kv_block_bytes(plan, 0), ab.amoeba_plan_kv_block_bytes(plan, 1)
    kv_src = [payload(kv_layers * src_pool_blocks * bb_s // 2) if kmask >> r & 1 else None
              for r in range(w.src_tp)]
    kv_dst = torch.empty(kv_layers * dst_pool_blocks * bb_d // 2, dtype=fdt, device="cuda")
    table_d = torch.from_numpy(table).cuda()
    lens_d = torch.from_numpy(lens).cuda()
    out_table = torch.empty_like(table_d)

    # When the whole cache does not fit beside its target (13B: 40 layers), the model's layers
    # are covered by several calls over the resident pools: full chunks of kv_layers and one
    # shorter call for the remainder, so that a step still moves every layer's worth of bytes.
    def calls_for(b):
        first = plan if b == bound else make_plan(kv_layers, b)
        calls = [first] * (w.n_layers // kv_layers)
        if w.n_layers % kv_layers:
            calls.append(make_plan(w.n_layers % kv_layers, b))
        return calls

    kv_calls = calls_for(bound)
    w_alg = 2 * dst_bytes
    kv_alg = 2 * total_blocks * bb_d * w.n_layers
    alg_bytes = w_alg + kv_alg

    def kv_step(calls):
        for p in calls:
            ab.amoeba_reshard_kv(p, kv_src, table_d, lens_d, kv_dst, out_table)

    def step(ev=None):
        ab.amoeba_reshard_weights(plan, w_src, w_dst)
        if ev is not None:
            ev[0].record()
        kv_step(kv_calls)
        if ev is not None:
            ev[1].record()

    for _ in range(args.warmup):
        step()
    rc, n_blocks = ab.amoeba_kv_status(plan)
    assert rc == ab.OK and n_blocks == total_blocks, (rc, n_blocks, ab.amoeba_last_error())

    # events sit on torch's current stream, which is the stream the binding hands to the library
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    first.record()
    for i in range(args.steps):
        step(evs[i])
    last.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kv_each = sorted(a.elapsed_time(b) for a, b in evs)
    kv_ms = sum(kv_each) / args.steps
    dev_ms = first.elapsed_time(last) / args.steps
    w_ms = dev_ms - kv_ms
    value = alg_bytes / (ms_per_step * 1e-3) / 1e9

    def timed_kv(calls, reps=5):
        for _ in range(2):
            kv_step(calls)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            kv_step(calls)
        b.record()
        torch.cuda.synchronize()
        return kv_alg * reps / (a.elapsed_time(b) * 1e-3) / 1e9

    # outside the timed region: the KV calls without the bound on the blocks in use (the grid
    # then covers the pool's capacity, four wavefronts per workgroup) ...
    other = calls_for(0 if bound else total_blocks)
    kv_other_gbps = timed_kv(other)
    for p in set(other):
        p.close()
    # ... and a plain streaming copy of the same access shape (one wavefront per 1 KiB tile, one
    # 16-byte vector per lane, non-temporal): the rate this GPU reaches on a copy, and a
    # transfer of known size for calibrating traffic counters
    copy_src = next(t for t in w_src if t is not None)
    copy_bytes = min(copy_src.numel(), w_dst.numel()) * 2 // 16 * 16
    for _ in range(2):
        ab.amoeba_copy_baseline(w_dst, copy_src, copy_bytes, 64, 1, 0, 1)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        ab.amoeba_copy_baseline(w_dst, copy_src, copy_bytes, 64, 1, 0, 1)
    c1.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * copy_bytes * 5 / (c0.elapsed_time(c1) * 1e-3) / 1e9

    kv_gbps = kv_alg / (kv_ms * 1e-3) / 1e9
    w_gbps = w_alg / (w_ms * 1e-3) / 1e9 if w_ms > 0 else None
    kgx, kgy, klanes, _ = ab.amoeba_plan_launch_shape(plan, ab.KERNEL_KV_REGROUP, 16)
    tune = (f"kv_blocks_bound={bound} in the shape" if bound else "no kv_blocks_bound") + \
        f" -> KV grid {kgx} x {kgy} workgroups of {klanes} lanes" + \
        (f"; overrides: {args.tune}" if args.tune else "")
    out = {
        "metric": "reshard throughput (read+write) of one TP transform, one target rank",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u16", "data": "synthetic",
        "pct_of_hbm_peak": round(100.0 * value / PEAK_HBM_GBPS, 2),
        "ms_per_tp_transform": round(ms_per_step, 4),
        "config": {"workload": f"{w.name}: TP{w.src_tp}->TP{w.dst_tp} rank {w.dst_rank}, "
                               f"{w.n_layers} layers, hidden {w.hidden}, {w.n_q_heads}q/"
                               f"{w.n_kv_heads}kv heads, d {w.head_dim}, ffn {w.ffn_dim}, "
                               f"{w.num_seqs} seqs / {int(lens.sum())} tokens / {total_blocks} "
                               f"blocks of {w.block_tokens}, KV layers resident {kv_layers} "
                               f"({len(kv_calls)} KV call(s) per step cover {w.n_layers} layers)",
                   "kv_layout": args.layout, "placement": args.placement,
                   "weights_alg_bytes": w_alg, "kv_alg_bytes": kv_alg,
                   "weights_ms": round(w_ms, 4), "weights_gbps": w_gbps and round(w_gbps, 1),
                   "kv_ms": round(kv_ms, 4), "kv_ms_median": round(kv_each[len(kv_each) // 2], 4),
                   "kv_ms_min": round(kv_each[0], 4), "kv_gbps": round(kv_gbps, 1),
                   "kv_gbps_without_bound": round(kv_other_gbps if bound else kv_gbps, 1),
                   "kv_gbps_with_bound": round(kv_gbps if bound else kv_other_gbps, 1),
                   "tune": tune,
                   "plain_copy_gbps": round(copy_gbps, 1), "plain_copy_bytes": copy_bytes},
        "roofline": {"bound": "hbm", "kernel": "kv_regroup_kernel", "achieved": round(kv_gbps, 1),
                     "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                     "frac": round(kv_gbps / PEAK_HBM_GBPS, 4), "traffic": None,
                     "alg_bytes_per_launch": kv_alg // len(kv_calls),   # mean over the launches
                     "launches_per_step": len(kv_calls),
                     "avg_launch_ms": round(kv_ms / len(kv_calls), 4)},
    }
    if w_gbps is not None and w_ms > kv_ms:
        # the weight kernel is the dominant one of this workload (few, short sequences)
        out["roofline"].update({"kernel": "reshard_weights_kernel", "achieved": round(w_gbps, 1),
                                "frac": round(w_gbps / PEAK_HBM_GBPS, 4),
                                "alg_bytes_per_launch": w_alg, "launches_per_step": 1,
                                "avg_launch_ms": round(w_ms, 4)})
    # HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, each calibrated on the plain copy kernel)
    # cannot be counted inside this process; they come from the committed rocprofv3 summary of
    # this workload, and only if that summary was taken on this build of the kernels
    summary = os.path.join(ROOT, "profiles", f"reshard_{w.name}_{args.layout}.txt")
    if os.path.exists(summary) and not args.tune and args.placement == "workload" and bound:
        text = open(summary).read()
        if f"kernel_sources_digest {kernel_sources_digest()}" in text:
            for line in text.splitlines():
                if line.startswith(f"traffic_bytes_per_launch {out['roofline']['kernel']}:"):
                    out["roofline"]["traffic"] = int(line.split(":")[1])
                    out["roofline"]["traffic_source"] = os.path.relpath(summary, ROOT)
        else:
            out["roofline"]["traffic_source"] = (
                f"{os.path.relpath(summary, ROOT)} was taken on another build of the kernels; "
                "not quoted")

    if args.graph:
        # the reshard calls only enqueue kernels (no allocation, no memset node), so a step can
        # be captured once and replayed
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        out["config"]["graph_replay_ms_per_step"] = round(
            (time.perf_counter() - g0) * 1e3 / args.steps, 4)
        rc, n_blocks = ab.amoeba_kv_status(plan)
        assert rc == ab.OK and n_blocks == total_blocks, (rc, n_blocks)

    for p in set(kv_calls) | {plan}:
        p.close()
    del w_src, w_dst, kv_src, kv_dst
    torch.cuda.empty_cache()
    if cpu_budget_s:
        out["cpu_baseline"] = cpu_baseline(w, lens, table, src_pool_blocks, dst_pool_blocks,
                                           lay_s, lay_d, cpu_budget_s)
        # the sample's rate applied to the whole transform (an extrapolation, not a measurement)
        out["cpu_baseline"]["extrapolated_ms_per_tp_transform"] = round(
            alg_bytes / (out["cpu_baseline"]["value"] * 1e9) * 1e3, 1)
    return out


def weights_padded(args):
    """Weight transformation TP1 <-> TP4 of the workload's model, dense layout against the
    padded partition-major FFN layout (2 MiB pages, T = 4).  Dense scale-up is the paper's
    "partial swap" (the kept partition is copied to the front); padded scale-up keeps a page
    range and copies only the attention part; scale-down gathers the other partitions.  For a
    mixture-of-experts workload the partitions are whole experts (TP1 EP1 <-> TP4 EP4)."""
    import torch

    from paper_2509_19729_amd import binding as ab
    from paper_2509_19729_amd import workloads as wl

    w = wl.WORKLOADS["llama7b" if args.workload == "all" else args.workload]
    T, page = 4, 2 << 20

    def shape(sp, dp):
        return ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim,
                             w.ffn_dim, elem_bytes=2, w_layout_src=sp, w_layout_dst=dp,
                             pad_max_tp=T, pad_page_bytes=page, n_experts=w.n_experts)

    def ffn_start(plan, side):
        """Bytes of a layer in front of the FFN part (attention tensors + their padding)."""
        if w.n_experts:
            return ab.amoeba_plan_expert_info(plan, side)[1]
        return ab.amoeba_plan_padded_info(plan, side)[1]

    def timed(plan, src, dst, part=ab.PART_ALL):
        for _ in range(args.warmup):
            ab.amoeba_reshard_weights_part(plan, src, dst, part)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            ab.amoeba_reshard_weights_part(plan, src, dst, part)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    def buf(nbytes):
        return torch.empty(nbytes // 2, dtype=torch.bfloat16, device="cuda").normal_(0.0, 0.02)

    res = {}
    # scale-up 1 -> 4, rank 1: dense (copy the whole shard) vs padded (attention part only)
    p_dense = ab.amoeba_plan(shape(0, 0), 1, 4, 1)
    src = [buf(ab.amoeba_plan_shard_bytes(p_dense, 0))]
    dst = buf(ab.amoeba_plan_shard_bytes(p_dense, 1))
    ms = timed(p_dense, src, dst)
    res["scale_up_dense_partial_swap"] = {"ms": round(ms, 4),
                                          "bytes_copied": ab.amoeba_plan_shard_bytes(p_dense, 1)}
    # the paper keeps the attention weights duplicated and swaps the FFN partition only
    # (Sec. 3.2): the same copy restricted to the FFN tensors
    ms_ffn = timed(p_dense, src, dst, ab.PART_FFN)
    t = [ab.amoeba_plan_tensor_info(p_dense, 1, x) for x in (ab.T_GATE, ab.T_UP, ab.T_DOWN)]
    ffn_bytes = sum(r * c for _, r, c, _ in t) * 2 * max(1, w.n_experts // 4) * w.n_layers
    res["scale_up_dense_partial_swap_ffn_only"] = {"ms": round(ms_ffn, 4), "bytes_copied": ffn_bytes}
    del src, dst
    torch.cuda.empty_cache()
    p_pad = ab.amoeba_plan(shape(1, 1), 1, 4, 1)
    rank, off, nbytes, src_layer = ab.amoeba_plan_ffn_view(p_pad)
    attn = ffn_start(p_pad, 1)
    # the FFN partitions stay where they are; only q/k/v/o are re-sliced (into a fresh buffer)
    a_src = [buf(ab.amoeba_plan_shard_bytes(p_pad, 0))]
    a_dst = buf(ab.amoeba_plan_shard_bytes(p_pad, 1))
    ms_attn = timed(p_pad, a_src, a_dst, ab.PART_ATTENTION)
    res["scale_up_padded"] = {"ms": round(ms_attn, 4), "bytes_copied": attn * w.n_layers,
                              "ffn_bytes_kept_in_place": nbytes * w.n_layers,
                              "ffn_bytes_released": (src_layer - nbytes - ffn_start(p_pad, 0))
                              * w.n_layers}
    del a_src, a_dst
    torch.cuda.empty_cache()
    # scale-down 4 -> 1: dense gather vs padded gather (both move the whole model)
    for name, sp in (("scale_down_dense", 0), ("scale_down_padded", 1)):
        plan = ab.amoeba_plan(shape(sp, sp), 4, 1, 0)
        src = [buf(ab.amoeba_plan_shard_bytes(plan, 0)) for _ in range(4)]
        dst = buf(ab.amoeba_plan_shard_bytes(plan, 1))
        ms = timed(plan, src, dst)
        nb = ab.amoeba_plan_shard_bytes(plan, 1)
        res[name] = {"ms": round(ms, 4), "bytes_copied": nb,
                     "gbps_read_plus_write": round(2 * nb / (ms * 1e-3) / 1e9, 1)}
        if sp and w.n_experts:
            _, _, tensor, slot = ab.amoeba_plan_expert_info(plan, 1)
            res["padding_overhead"] = round((slot - 3 * tensor) / (3 * tensor), 5)
        elif sp:
            info = ab.amoeba_plan_padded_info(plan, 1)
            res["padding_overhead"] = round((info[3] - info[2]) / info[2], 5)
        del src, dst
        torch.cuda.empty_cache()
        plan.close()
    up = res["scale_up_dense_partial_swap"]
    out = {"metric": "weight transformation TP1 <-> TP4, dense vs padded FFN layout", "unit": "ms",
           "value": res["scale_up_padded"]["ms"], "higher_is_better": False, "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "data": "synthetic", "dtype": "u16",
           "config": {"workload": f"{w.name}: {w.n_layers} layers, hidden {w.hidden}, ffn "
                                  f"{w.ffn_dim}" + (f" x {w.n_experts} experts" if w.n_experts else
                                                    f", T = {T}") + ", 2 MiB pages, target rank 1 / 0"},
           "results": res,
           "scale_up_time_saved": round(1 - res["scale_up_padded"]["ms"] / up["ms"], 4)}
    print(json.dumps(out), flush=True)


def overlap(args):
    """Sec. 3.1/3.2, Improvement 2, restated on one GPU: the transformation runs layer by layer
    on its own stream (default priority) while the instance keeps serving.  A synthetic serving
    step runs on the main stream: either compute-bound (bf16 GEMMs, prefill-like) or
    memory-bound (streaming 8 GiB, decode-like); n layers of weights + KV are resharded
    concurrently per step.  Reported: step time alone, reshard alone, both together."""
    import torch

    from paper_2509_19729_amd import binding as ab
    from paper_2509_19729_amd import workloads as wl

    w = wl.WORKLOADS["llama7b" if args.workload == "all" else args.workload]
    lens = wl.seq_lens(w)
    table, src_pool = wl.block_placement(w, lens)
    total = int(wl.blocks_per_seq(lens, w.block_tokens).sum())
    dst_pool = total + 64
    L = w.n_layers

    def plan_for(n):
        shape = ab.ModelShape(n, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim,
                              elem_bytes=2, kv_block_tokens=w.block_tokens, kv_layers=n,
                              num_seqs=w.num_seqs, max_blocks_per_seq=table.shape[1],
                              src_pool_blocks=src_pool, dst_pool_blocks=dst_pool,
                              kv_blocks_bound=total)
        p = ab.amoeba_plan(shape, w.src_tp, w.dst_tp, w.dst_rank)
        knobs = {k[len("TUNE_"):].lower(): getattr(ab, k) for k in dir(ab) if k.startswith("TUNE_")}
        for kv in filter(None, args.tune.split(",")):
            name, val = kv.split("=")
            ab.amoeba_plan_tune(p, knobs[name], int(val))
        return p

    full = plan_for(L)
    wmask, kmask = ab.amoeba_plan_src_rank_mask(full), ab.amoeba_plan_kv_rank_mask(full)
    sb, db = ab.amoeba_plan_shard_bytes(full, 0), ab.amoeba_plan_shard_bytes(full, 1)
    bs, bd = ab.amoeba_plan_kv_block_bytes(full, 0), ab.amoeba_plan_kv_block_bytes(full, 1)

    def buf(nbytes):
        return torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 256)

    w_src = [buf(sb) if wmask >> r & 1 else None for r in range(w.src_tp)]
    w_dst = torch.empty(db, dtype=torch.uint8, device="cuda")
    kv_src = [buf(L * src_pool * bs) if kmask >> r & 1 else None for r in range(w.src_tp)]
    kv_dst = torch.empty(L * dst_pool * bd, dtype=torch.uint8, device="cuda")
    table_d, lens_d = torch.from_numpy(table).cuda(), torch.from_numpy(lens).cuda()
    out_table = torch.empty_like(table_d)
    a = torch.randn(8192, 8192, dtype=torch.bfloat16, device="cuda")
    b = torch.randn(8192, 8192, dtype=torch.bfloat16, device="cuda")
    big = torch.empty(1 << 31, dtype=torch.float32, device="cuda")   # 8 GiB
    side = torch.cuda.Stream()

    def serve(kind):
        if kind == "gemm":
            for _ in range(8):
                torch.mm(a, b)
        else:
            big.add_(1.0)

    def reshard(plan, n, first):
        ws = [None if t is None else t[first * (sb // L):] for t in w_src]
        ks = [None if t is None else t[first * src_pool * bs:] for t in kv_src]
        ab.amoeba_reshard_weights(plan, ws, w_dst[first * (db // L):], stream=side)
        ab.amoeba_reshard_kv(plan, ks, table_d, lens_d, kv_dst[first * dst_pool * bd:], out_table,
                             stream=side)

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    rows = []
    for n in (1, 4, L):
        plan = full if n == L else plan_for(n)
        for kind in ("gemm", "stream"):
            t_serve = timed(lambda: serve(kind))
            t_resh = timed(lambda: reshard(plan, n, 0))

            def both():
                # the serving step is enqueued first: its kernels have few, long workgroups and
                # are dispatched at once; the reshard's short workgroups then take what is free
                side.wait_stream(torch.cuda.current_stream())
                serve(kind)
                reshard(plan, n, 0)
                torch.cuda.current_stream().wait_stream(side)
            t_both = timed(both)
            rows.append({"layers_per_step": n, "serving_step": kind,
                         "serve_alone_ms": round(t_serve, 4), "reshard_alone_ms": round(t_resh, 4),
                         "together_ms": round(t_both, 4),
                         "step_time_overhead": round(t_both / t_serve - 1, 4),
                         "hidden_fraction_of_reshard": round(
                             max(0.0, min(1.0, (t_serve + t_resh - t_both) / t_resh)), 4)})
    out = {"metric": "serving step time with n layers resharded concurrently on a side stream",
           "unit": "ms", "value": rows[0]["together_ms"], "higher_is_better": False, "n_gpus": 1,
           "steps": args.steps, "data": "synthetic", "dtype": "u16",
           "config": {"workload": f"{w.name}: TP{w.src_tp}->TP{w.dst_tp} rank {w.dst_rank}; serving "
                                  "step = 8 bf16 GEMMs 8192^3 (gemm) or one pass over 8 GiB (stream)"},
           "results": rows}
    print(json.dumps(out), flush=True)


def _instances(w, m):
    """Split the workload's sequences over m TP1 instances, each with its own pool (fullest
    instance at 90 % occupancy) and a table drawn from a seeded permutation."""
    import numpy as np

    from paper_2509_19729_amd import workloads as wl
    lens_all = wl.seq_lens(w)
    per = [lens_all[g::m] for g in range(m)]
    S = max(len(x) for x in per)
    per = [np.concatenate([x, np.zeros(S - len(x), np.int32)]) for x in per]
    nb = [wl.blocks_per_seq(x, w.block_tokens) for x in per]
    P = int(np.ceil(max(int(x.sum()) for x in nb) / 0.9))
    W = max(8, int(-(-max(int(x.max()) for x in nb) // 8) * 8))
    tables = []
    for g in range(m):
        rng = np.random.default_rng(2000 + w.index * 10 + g)
        ids = rng.permutation(P)[:int(nb[g].sum())]
        t = np.full((S, W), -1, dtype=np.int32)
        p = 0
        for i, n in enumerate(nb[g]):
            t[i, :n] = ids[p:p + n]
            p += int(n)
        tables.append(t)
    return per, nb, tables, S, P, W


def merge_naive(args):
    """The paper's base solution for the same m x TP1 -> TP m scenario (Sec. 3.1: migration and
    de-fragmentation on token-first blocks): the heads a worker keeps are strided pieces inside
    every block and must be compacted just like the heads it receives, so every block of every
    instance is regrouped into a second pool.  One step = one amoeba_merge_kv_base call (scan,
    table, migration pass over the remote instances' blocks, de-fragmentation pass over the
    local ones; the two passes are the two launches of the block gather in a kernel trace)."""
    import numpy as np
    import torch

    from paper_2509_19729_amd import binding as ab
    from paper_2509_19729_amd import workloads as wl

    w = wl.WORKLOADS["llama7b" if args.workload == "all" else args.workload]
    m, rank = args.instances, 1 % args.instances
    per, nb, tables, S, P, W = _instances(w, m)
    L = args.kv_layers or w.n_layers
    lay = {"hm": ab.KV_HEAD_MAJOR, "tm": ab.KV_TOKEN_MAJOR}
    layout = "tm-tm" if args.layout == "hm-hm" else args.layout   # the base solution is token-first
    lay_s, lay_d = (lay[x] for x in layout.split("-"))
    total_blocks = sum(int(x.sum()) for x in nb)
    local_blocks = int(nb[rank].sum())
    shape = ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim,
                          elem_bytes=2, kv_block_tokens=w.block_tokens, kv_layout_src=lay_s,
                          kv_layout_dst=lay_d, kv_layers=L, num_seqs=S, max_blocks_per_seq=W,
                          src_pool_blocks=P, dst_pool_blocks=total_blocks,
                          kv_blocks_bound=0 if args.no_bound else total_blocks)
    plan = ab.amoeba_plan(shape, 1, m, rank)
    bs, bd = ab.amoeba_plan_kv_block_bytes(plan, 0), ab.amoeba_plan_kv_block_bytes(plan, 1)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0xA30EBA10 + w.index)
    pools = []
    for g in range(m):
        t = torch.empty(L * P * bs // 2, dtype=torch.bfloat16, device="cuda")
        for a in range(0, t.numel(), 1 << 28):
            t[a:a + (1 << 28)].normal_(0.0, 0.02, generator=gen)
        pools.append(t)
    new_pool = torch.empty(L * total_blocks * bd // 2, dtype=torch.bfloat16, device="cuda")
    out_table = torch.empty((m * S, W), dtype=torch.int32, device="cuda")
    tabs_d = [torch.from_numpy(t).cuda() for t in tables]
    lens_d = [torch.from_numpy(x.astype(np.int32)).cuda() for x in per]
    def step():
        ab.amoeba_merge_kv_base(plan, pools, tabs_d, lens_d, new_pool, out_table,
                                0 if args.no_bound else local_blocks)

    for _ in range(args.warmup):
        step()
    rc, n = ab.amoeba_kv_status(plan)
    assert rc == ab.OK and n == total_blocks, (rc, n, ab.amoeba_last_error())
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    dev_ms = e0.elapsed_time(e1) / args.steps
    alg = 2 * total_blocks * bd * L
    out = {
        "metric": "base KV merge of Sec. 3.1 (migration + de-fragmentation into a second pool), "
                  "m x TP1 -> TP m, one target rank",
        "value": round(alg / (ms * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u16",
        "data": "synthetic",
        "config": {"workload": f"{w.name} KV cache: {m} x TP1 -> TP{m} rank {rank}, {L} layers, "
                               f"{m} x {S} seqs, {total_blocks} blocks of {w.block_tokens} "
                               f"({local_blocks} local), layout {layout}",
                   "alg_bytes": alg, "extra_device_memory_bytes": total_blocks * bd * L,
                   "device_ms": round(dev_ms, 4),
                   "migration_alg_bytes": 2 * (total_blocks - local_blocks) * bd * L,
                   "defragmentation_alg_bytes": 2 * local_blocks * bd * L},
    }
    plan.close()
    print(json.dumps(out), flush=True)


def merge_inplace(args):
    """m TP1 instances of the workload's model, each serving every m-th sequence of the
    workload with its own pool and table, merged in place into one TP=m instance; one step =
    one amoeba_merge_kv_inplace call for target rank 1 (header-centric layout, all layers)."""
    import numpy as np
    import torch

    from paper_2509_19729_amd import binding as ab
    from paper_2509_19729_amd import workloads as wl

    w = wl.WORKLOADS["llama7b" if args.workload == "all" else args.workload]
    m, rank = args.instances, 1 % args.instances
    per, nb, tables, S, P, W = _instances(w, m)
    L = args.kv_layers or w.n_layers
    # the scheduler that owns the tables knows how many blocks are remote; the library sizes
    # its grid by this bound instead of by the pool's capacity
    n_remote_host = sum(int(x.sum()) for g, x in enumerate(nb) if g != rank)
    shape = ab.ModelShape(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim,
                          elem_bytes=2, kv_block_tokens=w.block_tokens, kv_layers=L, num_seqs=S,
                          max_blocks_per_seq=W, src_pool_blocks=P, dst_pool_blocks=P * m,
                          kv_blocks_bound=0 if args.no_bound else n_remote_host)
    plan = ab.amoeba_plan(shape, 1, m, rank)
    assert ab.amoeba_plan_merge_factor(plan) == m
    bb = ab.amoeba_plan_kv_block_bytes(plan, 0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0xA30EBA10 + w.index)
    pools = []
    for g in range(m):
        t = torch.empty(L * P * bb // 2, dtype=torch.bfloat16, device="cuda")
        for a in range(0, t.numel(), 1 << 28):
            t[a:a + (1 << 28)].normal_(0.0, 0.02, generator=gen)
        pools.append(t)
    tabs_d = [torch.from_numpy(t).cuda() for t in tables]
    lens_d = [torch.from_numpy(x.astype(np.int32)).cuda() for x in per]
    out_table = torch.empty((m * S, W), dtype=torch.int32, device="cuda")
    remote = [None if g == rank else pools[g] for g in range(m)]

    def step():
        ab.amoeba_merge_kv_inplace(plan, pools[rank], remote, tabs_d, lens_d, out_table)

    for _ in range(args.warmup):
        step()
    rc, n_remote = ab.amoeba_merge_kv_status(plan)
    assert rc == ab.OK, ab.amoeba_last_error()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    dev_ms = e0.elapsed_time(e1) / args.steps
    sub = ab.amoeba_plan_kv_block_bytes(plan, 1)
    alg = 2 * n_remote * sub * L
    total_blocks = sum(int(x.sum()) for x in nb)
    out = {
        "metric": "in-place KV merge throughput (read+write), m x TP1 -> TP m, one target rank",
        "value": round(alg / (ms * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u16",
        "data": "synthetic",
        "config": {"workload": f"{w.name} KV cache: {m} x TP1 -> TP{m} rank {rank}, {L} layers, "
                               f"{w.n_kv_heads} kv heads, d {w.head_dim}, {m} x {S} seqs, "
                               f"{total_blocks} blocks of {w.block_tokens} in pools of {P} "
                               f"({bb} B blocks -> {sub} B blocks)",
                   "remote_blocks": n_remote, "alg_bytes": alg,
                   "bytes_an_out_of_place_regroup_moves": 2 * total_blocks * sub * L,
                   "extra_device_memory_bytes": 4 * (8 + (m * P + 1023) // 1024 + 1 + 2 * m * P)},
        "roofline": {"bound": "hbm", "kernel": "merge_copy_kernel",
                     "achieved": round(alg / (dev_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBPS,
                     "unit": "GB/s", "frac": round(alg / (dev_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                     "traffic": None, "alg_bytes_per_launch": alg,
                     "avg_launch_ms": round(dev_ms, 4)},
    }
    plan.close()
    print(json.dumps(out), flush=True)


def cpu_baseline(w, lens, table, src_pool_blocks, dst_pool_blocks, lay_s, lay_d, budget_s=12.0):
    """The oracle, single thread, on a bounded sample of the same workload: a few real-shape
    layers of weights and one layer of the whole KV table, repeated until about budget_s of CPU
    time have been spent (host speeds differ by an order of magnitude between boxes)."""
    import numpy as np

    import oracle
    from paper_2509_19729_amd import workloads as wl

    w_layers = max(1, min(w.n_layers, int(800e6 // max(1, _layer_bytes(w)))))
    m = oracle.Model(w_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn_dim)
    moe = oracle.Moe(w.n_experts) if w.n_experts else None
    n = oracle.moe_shard_elems(m, moe, False, w.src_tp) if moe else oracle.shard_elems(m, w.src_tp)
    src = [wl.random_bits(n, seed=11 + s) for s in range(w.src_tp)]
    dst = np.zeros(oracle.moe_shard_elems(m, moe, False, w.dst_tp) if moe
                   else oracle.shard_elems(m, w.dst_tp), dtype=np.uint16)
    kv = oracle.KV(kv_layers=1, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                   block_tokens=w.block_tokens, num_seqs=w.num_seqs,
                   max_blocks_per_seq=table.shape[1], src_pool_blocks=src_pool_blocks,
                   dst_pool_blocks=dst_pool_blocks, layout_src=lay_s, layout_dst=lay_d)
    be_s, be_d = oracle.kv_block_elems(kv, w.src_tp), oracle.kv_block_elems(kv, w.dst_tp)
    pools = [wl.random_bits(src_pool_blocks * be_s, seed=21 + s).reshape(1, src_pool_blocks, be_s)
             for s in range(w.src_tp)]
    dpool = np.zeros((1, dst_pool_blocks, be_d), dtype=np.uint16)

    t_w = t_kv = 0.0
    bytes_w = bytes_kv = 0
    reps = 0
    max_reps = 64
    while reps < max_reps and t_w + t_kv < budget_s:
        t0 = time.perf_counter()
        if moe:
            st, dst = oracle.reshard_weights_moe(m, moe, w.src_tp, w.dst_tp, w.dst_rank, src, dst)
        else:
            st, dst = oracle.reshard_weights(m, w.src_tp, w.dst_tp, w.dst_rank, src, dst)
        t_w += time.perf_counter() - t0
        assert st == oracle.OK
        bytes_w += 2 * dst.nbytes
        t0 = time.perf_counter()
        st, _, total = oracle.reshard_kv(kv, w.src_tp, w.dst_tp, w.dst_rank, pools, table, lens,
                                         dpool)
        t_kv += time.perf_counter() - t0
        assert st == oracle.OK
        bytes_kv += 2 * total * be_d * 2
        reps += 1
    gbps = (bytes_w + bytes_kv) / (t_w + t_kv) / 1e9
    return {"value": round(gbps, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{reps} x [{w_layers} real-shape layers of weights + 1 layer of the whole "
                      f"KV table]: weights {bytes_w / 1e9:.2f} GB r+w in {t_w:.2f} s, KV "
                      f"{bytes_kv / 1e9:.2f} GB r+w in {t_kv:.2f} s; single thread, g++ -O2",
            "host_cpus": os.cpu_count()}


def _layer_bytes(w):
    per = (2 * w.n_q_heads + 2 * w.n_kv_heads) * w.head_dim * w.hidden + \
        3 * w.hidden * w.ffn_dim * max(1, w.n_experts)
    return per * w.elem_bytes // w.dst_tp


if __name__ == "__main__":
    main()
