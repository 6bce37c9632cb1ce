"""Helpers for the GPU parity tests: move numpy payloads to the device as raw
bytes, call the library through its binding, bring results back.  No reshard
arithmetic lives here."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2509_19729_amd import binding as ab

_VIEW = {1: np.uint8, 2: np.int16, 4: np.int32}


def to_dev(a: np.ndarray) -> torch.Tensor:
    """Raw bytes of `a` on cuda:0 (as a signed view torch understands)."""
    return torch.from_numpy(np.ascontiguousarray(a).view(_VIEW[a.dtype.itemsize])).cuda()


def to_host(t: torch.Tensor, dtype) -> np.ndarray:
    return t.cpu().numpy().view(dtype)


def shape_from(m: oracle.Model, kv: oracle.KV | None = None) -> ab.ModelShape:
    s = ab.ModelShape(n_layers=m.n_layers, hidden=m.hidden, n_q_heads=m.n_q_heads,
                      n_kv_heads=m.n_kv_heads, head_dim=m.head_dim, ffn_dim=m.ffn_dim,
                      elem_bytes=m.elem_bytes)
    if kv is not None:
        assert kv.n_kv_heads == m.n_kv_heads and kv.head_dim == m.head_dim
        s.kv_block_tokens = kv.block_tokens
        s.kv_layout_src, s.kv_layout_dst = kv.layout_src, kv.layout_dst
        s.kv_layers = kv.kv_layers
        s.num_seqs, s.max_blocks_per_seq = kv.num_seqs, kv.max_blocks_per_seq
        s.src_pool_blocks, s.dst_pool_blocks = kv.src_pool_blocks, kv.dst_pool_blocks
    return s


def model_for_kv(kv: oracle.KV) -> oracle.Model:
    """A decoder shape carrying the KV geometry (weights unused by the KV tests)."""
    return oracle.Model(n_layers=kv.kv_layers, hidden=kv.n_kv_heads * kv.head_dim,
                        n_q_heads=kv.n_kv_heads, n_kv_heads=kv.n_kv_heads, head_dim=kv.head_dim,
                        ffn_dim=kv.n_kv_heads * 16, elem_bytes=kv.elem_bytes)


GUARD = 256  # elements of sentinel before and after a destination buffer


def gpu_reshard_weights(m: oracle.Model, k, kp, rp, src_np, tune=None, sentinel=0x5C):
    """Runs the library on device copies of src_np; returns (dst, guards_intact)."""
    dt = oracle.elem_dtype(m.elem_bytes)
    plan = ab.amoeba_plan(shape_from(m), k, kp, rp)
    for knob, val in (tune or {}).items():
        ab.amoeba_plan_tune(plan, knob, val)
    n = ab.amoeba_plan_shard_bytes(plan, 1) // m.elem_bytes
    src_dev = [None if a is None else to_dev(a) for a in src_np]
    buf = torch.full(((n + 2 * GUARD) * m.elem_bytes,), sentinel, dtype=torch.uint8, device="cuda")
    dst = buf[GUARD * m.elem_bytes:(GUARD + n) * m.elem_bytes]
    ab.amoeba_reshard_weights(plan, src_dev, dst)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    lo, hi = GUARD * m.elem_bytes, (GUARD + n) * m.elem_bytes
    intact = bool((host[:lo] == sentinel).all() and (host[hi:] == sentinel).all())
    plan.close()
    return host[lo:hi].view(dt), intact


def gpu_reshard_kv(kv: oracle.KV, k, kp, rp, src_pools_np, table_np, lens_np, tune=None,
                   sentinel=0xA7, bound=0):
    """Returns (status, dst_pool, dst_table, total, guards_intact); the destination pool
    starts filled with `sentinel` bytes so untouched blocks can be compared too.  `bound`
    goes into the shape's kv_blocks_bound."""
    dt = oracle.elem_dtype(kv.elem_bytes)
    shape = shape_from(model_for_kv(kv), kv)
    shape.kv_blocks_bound = bound
    plan = ab.amoeba_plan(shape, k, kp, rp)
    for knob, val in (tune or {}).items():
        ab.amoeba_plan_tune(plan, knob, val)
    bb = ab.amoeba_plan_kv_block_bytes(plan, 1)
    n_bytes = kv.kv_layers * kv.dst_pool_blocks * bb
    g = GUARD * 4
    buf = torch.full((n_bytes + 2 * g,), sentinel, dtype=torch.uint8, device="cuda")
    dst = buf[g:g + n_bytes]
    src_dev = [None if a is None else to_dev(a) for a in src_pools_np]
    table_dev = torch.from_numpy(np.ascontiguousarray(table_np, dtype=np.int32)).cuda()
    lens_dev = torch.from_numpy(np.ascontiguousarray(lens_np, dtype=np.int32)).cuda()
    out_table = torch.full((kv.num_seqs, kv.max_blocks_per_seq), -9, dtype=torch.int32,
                           device="cuda")
    ab.amoeba_reshard_kv(plan, src_dev, table_dev, lens_dev, dst, out_table)
    st, total = ab.amoeba_kv_status(plan)
    host = buf.cpu().numpy()
    intact = bool((host[:g] == sentinel).all() and (host[g + n_bytes:] == sentinel).all())
    pool = host[g:g + n_bytes].view(dt).reshape(kv.kv_layers, kv.dst_pool_blocks, -1)
    plan.close()
    return st, pool, out_table.cpu().numpy(), total, intact


def sentinel_elem(elem_bytes, byte):
    return int.from_bytes(bytes([byte]) * elem_bytes, "little")
