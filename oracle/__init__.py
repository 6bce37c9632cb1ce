"""CPU oracle for the TP=k -> TP=k' reshard (TEST INFRASTRUCTURE ONLY).

Thin ctypes driver around ``amoeba_oracle.cpp`` operating on numpy arrays in
host memory.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product
package never does.  The arithmetic lives in the C++ file, which cites the
paper passages it follows (Sec. 2.2, Sec. 3.1 head-range rule and layouts,
Sec. 3.2 Eq. (1)).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "amoeba_oracle.cpp")
_LIB = os.path.join(_HERE, "libamoeba_oracle.so")

HEAD_MAJOR = 0
TOKEN_MAJOR = 1

OK, ERR_ARG, ERR_OVERFLOW, ERR_BLOCK_ID = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with g++ -O2 (no threads, no intrinsics)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "amoeba_oracle.h")))
    if force or stale:
        subprocess.check_call(
            ["g++", "-std=c++17", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


class _Model(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim",
                 "elem_bytes")]


class _KV(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("kv_layers", "n_kv_heads", "head_dim", "elem_bytes", "block_tokens",
                 "layout_src", "layout_dst", "num_seqs", "max_blocks_per_seq")] + \
               [("src_pool_blocks", ctypes.c_int64), ("dst_pool_blocks", ctypes.c_int64)]


class _Pad(ctypes.Structure):
    _fields_ = [("max_tp", ctypes.c_int32), ("src_padded", ctypes.c_int32),
                ("dst_padded", ctypes.c_int32), ("page_bytes", ctypes.c_int64)]


class _Moe(ctypes.Structure):
    _fields_ = [("n_experts", ctypes.c_int32), ("src_padded", ctypes.c_int32),
                ("dst_padded", ctypes.c_int32), ("page_bytes", ctypes.c_int64)]


@dataclass(frozen=True)
class Moe:
    """Expert-wise FFN layout (Sec. 3.2, EP discussion); Model.ffn_dim is one expert's size."""
    n_experts: int
    page_bytes: int = 0
    src_padded: bool = False
    dst_padded: bool = False

    def _c(self):
        return _Moe(self.n_experts, int(self.src_padded), int(self.dst_padded), self.page_bytes)


@dataclass(frozen=True)
class Pad:
    """Padded FFN layout parameters (Sec. 3.2, Improvement 1)."""
    max_tp: int
    page_bytes: int
    src_padded: bool = False
    dst_padded: bool = True

    def _c(self):
        return _Pad(self.max_tp, int(self.src_padded), int(self.dst_padded), self.page_bytes)


@dataclass(frozen=True)
class Model:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    elem_bytes: int = 2

    def _c(self):
        return _Model(self.n_layers, self.hidden, self.n_q_heads, self.n_kv_heads, self.head_dim,
                      self.ffn_dim, self.elem_bytes)


@dataclass(frozen=True)
class KV:
    kv_layers: int
    n_kv_heads: int
    head_dim: int
    block_tokens: int
    num_seqs: int
    max_blocks_per_seq: int
    src_pool_blocks: int
    dst_pool_blocks: int
    layout_src: int = HEAD_MAJOR
    layout_dst: int = HEAD_MAJOR
    elem_bytes: int = 2

    def _c(self):
        return _KV(self.kv_layers, self.n_kv_heads, self.head_dim, self.elem_bytes,
                   self.block_tokens, self.layout_src, self.layout_dst, self.num_seqs,
                   self.max_blocks_per_seq, self.src_pool_blocks, self.dst_pool_blocks)


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.ao_shard_elems.restype = ctypes.c_int64
        L.ao_shard_elems.argtypes = [ctypes.POINTER(_Model), ctypes.c_int]
        L.ao_kv_block_elems.restype = ctypes.c_int64
        L.ao_kv_block_elems.argtypes = [ctypes.POINTER(_KV), ctypes.c_int]
        L.ao_reshard_weights.restype = ctypes.c_int
        L.ao_reshard_weights.argtypes = [ctypes.POINTER(_Model), ctypes.c_int, ctypes.c_int,
                                         ctypes.c_int, ctypes.POINTER(ctypes.c_void_p),
                                         ctypes.c_void_p]
        L.ao_reshard_kv.restype = ctypes.c_int
        L.ao_reshard_kv.argtypes = [ctypes.POINTER(_KV), ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.POINTER(ctypes.c_int64)]
        L.ao_merge_kv_inplace.restype = ctypes.c_int
        L.ao_merge_kv_inplace.argtypes = [ctypes.POINTER(_KV), ctypes.c_int, ctypes.c_int,
                                          ctypes.c_int, ctypes.c_void_p,
                                          ctypes.POINTER(ctypes.c_void_p),
                                          ctypes.POINTER(ctypes.c_void_p),
                                          ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p,
                                          ctypes.POINTER(ctypes.c_int64)]
        L.ao_merge_kv_base.restype = ctypes.c_int
        L.ao_merge_kv_base.argtypes = [ctypes.POINTER(_KV), ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, ctypes.POINTER(ctypes.c_void_p),
                                       ctypes.POINTER(ctypes.c_void_p),
                                       ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64),
                                       ctypes.POINTER(ctypes.c_int64)]
        L.ao_padded_shard_elems.restype = ctypes.c_int64
        L.ao_padded_shard_elems.argtypes = [ctypes.POINTER(_Model), ctypes.POINTER(_Pad),
                                            ctypes.c_int]
        L.ao_padded_geometry.restype = ctypes.c_int
        L.ao_padded_geometry.argtypes = [ctypes.POINTER(_Model), ctypes.POINTER(_Pad),
                                         ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]
        L.ao_reshard_weights_padded.restype = ctypes.c_int
        L.ao_reshard_weights_padded.argtypes = [ctypes.POINTER(_Model), ctypes.POINTER(_Pad),
                                                ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p]
        L.ao_moe_shard_elems.restype = ctypes.c_int64
        L.ao_moe_shard_elems.argtypes = [ctypes.POINTER(_Model), ctypes.POINTER(_Moe),
                                         ctypes.c_int, ctypes.c_int]
        L.ao_moe_geometry.restype = ctypes.c_int
        L.ao_moe_geometry.argtypes = [ctypes.POINTER(_Model), ctypes.POINTER(_Moe), ctypes.c_int,
                                      ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]
        L.ao_reshard_weights_moe.restype = ctypes.c_int
        L.ao_reshard_weights_moe.argtypes = [ctypes.POINTER(_Model), ctypes.POINTER(_Moe),
                                             ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                             ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p]
        _lib = L
    return _lib


_DT = {1: np.uint8, 2: np.uint16, 4: np.uint32}


def elem_dtype(elem_bytes: int):
    return _DT[elem_bytes]


def shard_elems(m: Model, tp: int) -> int:
    return int(lib().ao_shard_elems(ctypes.byref(m._c()), tp))


def kv_block_elems(c: KV, tp: int) -> int:
    return int(lib().ao_kv_block_elems(ctypes.byref(c._c()), tp))


def _ptr_array(arrs, n, dtype):
    out = (ctypes.c_void_p * n)()
    keep = []
    for i in range(n):
        a = arrs[i] if i < len(arrs) else None
        if a is None:
            out[i] = None
        else:
            assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], "oracle wants contiguous arrays"
            keep.append(a)
            out[i] = a.ctypes.data
    return out, keep


def reshard_weights(m: Model, src_tp: int, dst_tp: int, dst_rank: int, src_shards, dst=None):
    """src_shards: list of src_tp 1-D arrays (opaque elements) or None.  Returns (status, dst)."""
    dt = elem_dtype(m.elem_bytes)
    n = shard_elems(m, dst_tp)
    if dst is None:
        dst = np.zeros(max(n, 0), dtype=dt)
    ptrs, _keep = _ptr_array(src_shards, max(src_tp, 1), dt)
    st = lib().ao_reshard_weights(ctypes.byref(m._c()), src_tp, dst_tp, dst_rank, ptrs,
                                  dst.ctypes.data)
    return int(st), dst


def reshard_kv(c: KV, src_tp: int, dst_tp: int, dst_rank: int, src_pools, src_table, seq_lens,
               dst_pool, dst_table=None):
    """src_pools: list of src_tp arrays [kv_layers, src_pool_blocks, block_elems] or None.
    dst_pool is written in place.  Returns (status, dst_table, total_blocks)."""
    dt = elem_dtype(c.elem_bytes)
    src_table = np.ascontiguousarray(src_table, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    if dst_table is None:
        dst_table = np.full((c.num_seqs, c.max_blocks_per_seq), -7, dtype=np.int32)
    assert dst_table.dtype == np.int32 and dst_table.flags["C_CONTIGUOUS"]
    assert dst_pool.dtype == dt and dst_pool.flags["C_CONTIGUOUS"]
    ptrs, _keep = _ptr_array(src_pools, max(src_tp, 1), dt)
    total = ctypes.c_int64(-1)
    st = lib().ao_reshard_kv(ctypes.byref(c._c()), src_tp, dst_tp, dst_rank, ptrs,
                             src_table.ctypes.data, seq_lens.ctypes.data, dst_pool.ctypes.data,
                             dst_table.ctypes.data, ctypes.byref(total))
    return int(st), dst_table, int(total.value)


def merge_kv_inplace(c: KV, src_tp: int, m: int, dst_rank: int, local_pool, remote_pools,
                     src_tables, seq_lens, dst_table=None):
    """In-place merge of m instances (header-centric).  local_pool [kv_layers, P, block(src_tp)]
    is modified in place; remote_pools: m arrays (entry dst_rank % m may be None); src_tables,
    seq_lens: m arrays each.  Returns (status, dst_table [m*S, W], remote_blocks)."""
    dt = elem_dtype(c.elem_bytes)
    assert local_pool.dtype == dt and local_pool.flags["C_CONTIGUOUS"]
    tabs = [np.ascontiguousarray(t, dtype=np.int32) for t in src_tables]
    lens = [np.ascontiguousarray(x, dtype=np.int32) for x in seq_lens]
    if dst_table is None:
        dst_table = np.full((m * c.num_seqs, c.max_blocks_per_seq), -7, dtype=np.int32)
    pools, _k1 = _ptr_array(remote_pools, max(m, 1), dt)
    tptr, _k2 = _ptr_array(tabs, max(m, 1), np.int32)
    lptr, _k3 = _ptr_array(lens, max(m, 1), np.int32)
    n = ctypes.c_int64(-1)
    st = lib().ao_merge_kv_inplace(ctypes.byref(c._c()), src_tp, m, dst_rank,
                                   local_pool.ctypes.data, pools, tptr, lptr,
                                   dst_table.ctypes.data, ctypes.byref(n))
    return int(st), dst_table, int(n.value)


def merge_kv_base(c: KV, src_tp: int, m: int, dst_rank: int, pools, src_tables, seq_lens,
                  new_pool, dst_table=None):
    """The base solution of Sec. 3.1 (migration, then de-fragmentation, into new_pool, which is
    written in place).  pools: m arrays [kv_layers, P, block(src_tp)]; src_tables, seq_lens:
    m arrays each.  Returns (status, dst_table [m*S, W], migrated_blocks, defrag_blocks)."""
    dt = elem_dtype(c.elem_bytes)
    assert new_pool.dtype == dt and new_pool.flags["C_CONTIGUOUS"]
    tabs = [np.ascontiguousarray(t, dtype=np.int32) for t in src_tables]
    lens = [np.ascontiguousarray(x, dtype=np.int32) for x in seq_lens]
    if dst_table is None:
        dst_table = np.full((m * c.num_seqs, c.max_blocks_per_seq), -7, dtype=np.int32)
    pptr, _k1 = _ptr_array(pools, max(m, 1), dt)
    tptr, _k2 = _ptr_array(tabs, max(m, 1), np.int32)
    lptr, _k3 = _ptr_array(lens, max(m, 1), np.int32)
    mig, dfr = ctypes.c_int64(-1), ctypes.c_int64(-1)
    st = lib().ao_merge_kv_base(ctypes.byref(c._c()), src_tp, m, dst_rank, pptr, tptr, lptr,
                                new_pool.ctypes.data, dst_table.ctypes.data, ctypes.byref(mig),
                                ctypes.byref(dfr))
    return int(st), dst_table, int(mig.value), int(dfr.value)


def padded_shard_elems(m: Model, pad: Pad, tp: int) -> int:
    return int(lib().ao_padded_shard_elems(ctypes.byref(m._c()), ctypes.byref(pad._c()), tp))


def padded_geometry(m: Model, pad: Pad, tp: int):
    """(attn, attn_padded, part, part_padded, stride, layer) in elements at TP=tp."""
    out = (ctypes.c_int64 * 6)()
    st = lib().ao_padded_geometry(ctypes.byref(m._c()), ctypes.byref(pad._c()), tp, out)
    assert st == OK
    return tuple(int(x) for x in out)


def reshard_weights_padded(m: Model, pad: Pad, src_tp: int, dst_tp: int, dst_rank: int,
                           src_shards, dst=None):
    """Reshard with either side in the padded layout.  Returns (status, dst)."""
    dt = elem_dtype(m.elem_bytes)
    n = padded_shard_elems(m, pad, dst_tp) if pad.dst_padded else shard_elems(m, dst_tp)
    if dst is None:
        dst = np.full(max(n, 0), 0xEE, dtype=dt)
    ptrs, _keep = _ptr_array(src_shards, max(src_tp, 1), dt)
    st = lib().ao_reshard_weights_padded(ctypes.byref(m._c()), ctypes.byref(pad._c()), src_tp,
                                         dst_tp, dst_rank, ptrs, dst.ctypes.data)
    return int(st), dst


def moe_shard_elems(m: Model, x: Moe, padded: bool, tp: int) -> int:
    return int(lib().ao_moe_shard_elems(ctypes.byref(m._c()), ctypes.byref(x._c()), int(padded), tp))


def moe_geometry(m: Model, x: Moe, padded: bool, tp: int):
    """(experts per rank, first expert offset, tensor, expert stride, layer) in elements."""
    out = (ctypes.c_int64 * 5)()
    st = lib().ao_moe_geometry(ctypes.byref(m._c()), ctypes.byref(x._c()), int(padded), tp, out)
    assert st == OK
    return tuple(int(v) for v in out)


def reshard_weights_moe(m: Model, x: Moe, src_tp: int, dst_tp: int, dst_rank: int, src_shards,
                        dst=None):
    """Mixture-of-experts reshard (attention by head, whole experts).  Returns (status, dst)."""
    dt = elem_dtype(m.elem_bytes)
    n = moe_shard_elems(m, x, x.dst_padded, dst_tp)
    if dst is None:
        dst = np.full(max(n, 0), 0xEE, dtype=dt)
    ptrs, _keep = _ptr_array(src_shards, max(src_tp, 1), dt)
    st = lib().ao_reshard_weights_moe(ctypes.byref(m._c()), ctypes.byref(x._c()), src_tp, dst_tp,
                                      dst_rank, ptrs, dst.ctypes.data)
    return int(st), dst
