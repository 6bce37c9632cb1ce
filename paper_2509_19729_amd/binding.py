"""ctypes binding of libamoeba.so: same names as the C ABI, argument marshalling only.

Device buffers are torch tensors (torch is used for device memory and streams,
nothing else); every step of the reshard runs in the library's HIP kernels.
There is no fallback: if the built library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, fields

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libamoeba.so")

KV_HEAD_MAJOR = 0
KV_TOKEN_MAJOR = 1

W_DENSE = 0
W_FFN_PADDED = 1

OK, ERR_INVALID_ARG, ERR_HIP, ERR_OVERFLOW, ERR_BLOCK_ID = 0, 1, 2, 3, 4

T_Q, T_K, T_V, T_O, T_GATE, T_UP, T_DOWN = range(7)

PART_ALL, PART_ATTENTION, PART_FFN = 0, 1, 2

# include/amoeba_measure.h
TUNE_W_GRID, TUNE_W_UNROLL, TUNE_W_THREADS, TUNE_KV_GRID, TUNE_KV_UNROLL, TUNE_KV_THREADS, \
    TUNE_NONTEMPORAL, TUNE_KV_STAGED, TUNE_KV_BLOCKS_HINT, TUNE_KV_SMALL_TABLE = range(10)
KERNEL_WEIGHTS, KERNEL_KV_REGROUP, KERNEL_MERGE_COPY = 0, 1, 2

MAX_TP = 16

# every symbol include/amoeba.h declares
EXPORTS = [
    "amoeba_plan", "amoeba_plan_destroy", "amoeba_reshard_weights", "amoeba_reshard_weights_part",
    "amoeba_reshard_kv", "amoeba_reshard_kv_static", "amoeba_kv_status", "amoeba_plan_shard_bytes",
    "amoeba_plan_kv_block_bytes", "amoeba_plan_src_rank_mask", "amoeba_plan_kv_rank_mask",
    "amoeba_plan_tensor_info", "amoeba_plan_kv_stride_order", "amoeba_plan_num_segments",
    "amoeba_plan_segment", "amoeba_last_error", "amoeba_merge_kv_inplace", "amoeba_merge_kv_base",
    "amoeba_merge_kv_status", "amoeba_plan_merge_factor", "amoeba_plan_padded_info",
    "amoeba_plan_ffn_view", "amoeba_plan_expert_info",
]
# every symbol include/amoeba_measure.h declares
MEASURE_EXPORTS = ["amoeba_plan_tune", "amoeba_plan_launch_shape", "amoeba_copy_baseline"]


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim",
                 "elem_bytes", "kv_block_tokens", "kv_layout_src", "kv_layout_dst", "kv_layers",
                 "num_seqs", "max_blocks_per_seq")] + \
               [("src_pool_blocks", ctypes.c_int64), ("dst_pool_blocks", ctypes.c_int64),
                ("w_layout_src", ctypes.c_int32), ("w_layout_dst", ctypes.c_int32),
                ("pad_max_tp", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("pad_page_bytes", ctypes.c_int64), ("kv_blocks_bound", ctypes.c_int64)]


@dataclass
class ModelShape:
    """Mirror of amoeba_model_shape."""
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    elem_bytes: int = 2
    kv_block_tokens: int = 16
    kv_layout_src: int = KV_HEAD_MAJOR
    kv_layout_dst: int = KV_HEAD_MAJOR
    kv_layers: int = 1
    num_seqs: int = 0
    max_blocks_per_seq: int = 0
    src_pool_blocks: int = 0
    dst_pool_blocks: int = 0
    w_layout_src: int = 0
    w_layout_dst: int = 0
    pad_max_tp: int = 0
    n_experts: int = 0
    pad_page_bytes: int = 0
    kv_blocks_bound: int = 0

    def _c(self) -> _Shape:
        return _Shape(*[getattr(self, f.name) for f in fields(self)])


_lib = None


def lib() -> ctypes.CDLL:
    """Load libamoeba.so (after torch, so both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is not built; run `python -m paper_2509_19729_amd.build` "
            "(there is no CPU fallback)")
    import torch  # noqa: F401  (loads libamdhip64 first)
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    L.amoeba_plan.restype = vp
    L.amoeba_plan.argtypes = [ctypes.POINTER(_Shape), i32, i32, i32]
    L.amoeba_plan_destroy.restype = None
    L.amoeba_plan_destroy.argtypes = [vp]
    L.amoeba_reshard_weights.restype = i32
    L.amoeba_reshard_weights.argtypes = [vp, ctypes.POINTER(vp), vp, vp]
    L.amoeba_reshard_weights_part.restype = i32
    L.amoeba_reshard_weights_part.argtypes = [vp, ctypes.POINTER(vp), vp, i32, vp]
    L.amoeba_reshard_kv.restype = i32
    L.amoeba_reshard_kv.argtypes = [vp, ctypes.POINTER(vp), vp, vp, vp, vp, vp]
    L.amoeba_reshard_kv_static.restype = i32
    L.amoeba_reshard_kv_static.argtypes = [vp, ctypes.POINTER(vp), vp, vp, vp, vp, vp]
    L.amoeba_kv_status.restype = i32
    L.amoeba_kv_status.argtypes = [vp, vp, ctypes.POINTER(i64)]
    L.amoeba_plan_shard_bytes.restype = ctypes.c_size_t
    L.amoeba_plan_shard_bytes.argtypes = [vp, i32]
    L.amoeba_plan_kv_block_bytes.restype = ctypes.c_size_t
    L.amoeba_plan_kv_block_bytes.argtypes = [vp, i32]
    L.amoeba_plan_src_rank_mask.restype = ctypes.c_uint32
    L.amoeba_plan_src_rank_mask.argtypes = [vp]
    L.amoeba_plan_kv_rank_mask.restype = ctypes.c_uint32
    L.amoeba_plan_kv_rank_mask.argtypes = [vp]
    L.amoeba_plan_tensor_info.restype = i32
    L.amoeba_plan_tensor_info.argtypes = [vp, i32, i32] + [ctypes.POINTER(i64)] * 4
    L.amoeba_plan_kv_stride_order.restype = i32
    L.amoeba_plan_kv_stride_order.argtypes = [vp, i32, ctypes.POINTER(i64)]
    L.amoeba_plan_num_segments.restype = i32
    L.amoeba_plan_num_segments.argtypes = [vp]
    L.amoeba_plan_segment.restype = i32
    L.amoeba_plan_segment.argtypes = [vp, i32, ctypes.POINTER(i64)]
    L.amoeba_plan_tune.restype = i32
    L.amoeba_plan_tune.argtypes = [vp, i32, i32]
    L.amoeba_plan_launch_shape.restype = i32
    L.amoeba_plan_launch_shape.argtypes = [vp, i32, i32, ctypes.POINTER(i64)]
    L.amoeba_copy_baseline.restype = i32
    L.amoeba_copy_baseline.argtypes = [vp, vp, ctypes.c_size_t, i32, i32, i32, i32, vp]
    L.amoeba_merge_kv_inplace.restype = i32
    L.amoeba_merge_kv_inplace.argtypes = [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                          ctypes.POINTER(vp), vp, vp]
    L.amoeba_merge_kv_base.restype = i32
    L.amoeba_merge_kv_base.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                       ctypes.POINTER(vp), vp, vp, i64, vp]
    L.amoeba_merge_kv_status.restype = i32
    L.amoeba_merge_kv_status.argtypes = [vp, vp, ctypes.POINTER(i64)]
    L.amoeba_plan_merge_factor.restype = i32
    L.amoeba_plan_merge_factor.argtypes = [vp]
    L.amoeba_plan_padded_info.restype = i32
    L.amoeba_plan_padded_info.argtypes = [vp, i32, ctypes.POINTER(i64)]
    L.amoeba_plan_expert_info.restype = i32
    L.amoeba_plan_expert_info.argtypes = [vp, i32, ctypes.POINTER(i64)]
    L.amoeba_plan_ffn_view.restype = i32
    L.amoeba_plan_ffn_view.argtypes = [vp, ctypes.POINTER(i64)]
    L.amoeba_last_error.restype = ctypes.c_char_p
    L.amoeba_last_error.argtypes = []
    _lib = L
    return L


class AmoebaError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"amoeba error {code}: {text}")
        self.code = code


def amoeba_last_error() -> str:
    return lib().amoeba_last_error().decode()


def _ptr(x) -> int:
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return x.ctypes.data


def _stream_handle(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Plan:
    """Owns an amoeba_plan_t*."""

    def __init__(self, handle: int, shape: ModelShape, src_tp: int, dst_tp: int, dst_rank: int):
        self.handle, self.shape = handle, shape
        self.src_tp, self.dst_tp, self.dst_rank = src_tp, dst_tp, dst_rank

    def close(self):
        if self.handle:
            lib().amoeba_plan_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def amoeba_plan(shape: ModelShape, src_tp: int, dst_tp: int, dst_rank: int) -> Plan:
    h = lib().amoeba_plan(ctypes.byref(shape._c()), src_tp, dst_tp, dst_rank)
    if not h:
        raise AmoebaError(ERR_INVALID_ARG, amoeba_last_error())
    return Plan(h, shape, src_tp, dst_tp, dst_rank)


def amoeba_plan_destroy(plan: Plan) -> None:
    plan.close()


def _ptr_array(items, n):
    arr = (ctypes.c_void_p * max(n, 1))()
    for i in range(n):
        arr[i] = _ptr(items[i]) if i < len(items) else 0
    return arr


def amoeba_reshard_weights(plan: Plan, src_shards, dst, stream=None, check: bool = True) -> int:
    rc = lib().amoeba_reshard_weights(plan.handle, _ptr_array(src_shards, plan.src_tp), _ptr(dst),
                                      _stream_handle(stream))
    if check and rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return rc


def amoeba_reshard_weights_part(plan: Plan, src_shards, dst, part: int, stream=None,
                                check: bool = True) -> int:
    rc = lib().amoeba_reshard_weights_part(plan.handle, _ptr_array(src_shards, plan.src_tp),
                                           _ptr(dst), part, _stream_handle(stream))
    if check and rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return rc


def amoeba_reshard_kv(plan: Plan, src_blocks, src_block_tables, seq_lens, dst_blocks,
                      dst_block_tables, stream=None, check: bool = True) -> int:
    rc = lib().amoeba_reshard_kv(plan.handle, _ptr_array(src_blocks, plan.src_tp),
                                 _ptr(src_block_tables), _ptr(seq_lens), _ptr(dst_blocks),
                                 _ptr(dst_block_tables), _stream_handle(stream))
    if check and rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return rc


def amoeba_reshard_kv_static(plan: Plan, src_blocks, src_block_tables, seq_lens, dst_blocks,
                             dst_block_tables, stream=None, check: bool = True) -> int:
    rc = lib().amoeba_reshard_kv_static(plan.handle, _ptr_array(src_blocks, plan.src_tp),
                                        _ptr(src_block_tables), _ptr(seq_lens), _ptr(dst_blocks),
                                        _ptr(dst_block_tables), _stream_handle(stream))
    if check and rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return rc


def amoeba_kv_status(plan: Plan, stream=None):
    """Synchronises the stream; returns (status, total_blocks)."""
    total = ctypes.c_int64(0)
    rc = lib().amoeba_kv_status(plan.handle, _stream_handle(stream), ctypes.byref(total))
    return rc, int(total.value)


def amoeba_plan_shard_bytes(plan: Plan, side: int) -> int:
    return int(lib().amoeba_plan_shard_bytes(plan.handle, side))


def amoeba_plan_kv_block_bytes(plan: Plan, side: int) -> int:
    return int(lib().amoeba_plan_kv_block_bytes(plan.handle, side))


def amoeba_plan_src_rank_mask(plan: Plan) -> int:
    return int(lib().amoeba_plan_src_rank_mask(plan.handle))


def amoeba_plan_kv_rank_mask(plan: Plan) -> int:
    return int(lib().amoeba_plan_kv_rank_mask(plan.handle))


def amoeba_plan_tensor_info(plan: Plan, side: int, tensor: int):
    """(elem_off, rows, cols, layer_elems)"""
    v = [ctypes.c_int64(0) for _ in range(4)]
    rc = lib().amoeba_plan_tensor_info(plan.handle, side, tensor, *[ctypes.byref(x) for x in v])
    if rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return tuple(int(x.value) for x in v)


def amoeba_plan_kv_stride_order(plan: Plan, side: int):
    """(stride_head, stride_kv, stride_token, stride_d, block_elems) in elements."""
    out = (ctypes.c_int64 * 5)()
    rc = lib().amoeba_plan_kv_stride_order(plan.handle, side, out)
    if rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return tuple(int(x) for x in out)


def amoeba_plan_num_segments(plan: Plan) -> int:
    return int(lib().amoeba_plan_num_segments(plan.handle))


def amoeba_plan_segment(plan: Plan, index: int):
    """(src_rank, src_byte_off, src_pitch, dst_byte_off, dst_pitch, rows, run_bytes)"""
    out = (ctypes.c_int64 * 7)()
    rc = lib().amoeba_plan_segment(plan.handle, index, out)
    if rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return tuple(int(x) for x in out)


def amoeba_plan_tune(plan: Plan, knob: int, value: int) -> None:
    rc = lib().amoeba_plan_tune(plan.handle, knob, value)
    if rc != OK:
        raise AmoebaError(rc, amoeba_last_error())


def amoeba_plan_launch_shape(plan: Plan, kernel: int, align_bytes: int = 16):
    """(grid.x, grid.y, lanes per workgroup, work items per grid.y slice)"""
    out = (ctypes.c_int64 * 4)()
    rc = lib().amoeba_plan_launch_shape(plan.handle, kernel, align_bytes, out)
    if rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return tuple(int(x) for x in out)


def amoeba_copy_baseline(dst, src, nbytes: int, threads: int = 64, unroll: int = 1, grid: int = 0,
                         nontemporal: int = 1, stream=None) -> None:
    rc = lib().amoeba_copy_baseline(_ptr(dst), _ptr(src), nbytes, threads, unroll, grid,
                                    nontemporal, _stream_handle(stream))
    if rc != OK:
        raise AmoebaError(rc, amoeba_last_error())


def amoeba_plan_merge_factor(plan: Plan) -> int:
    return int(lib().amoeba_plan_merge_factor(plan.handle))


def amoeba_merge_kv_inplace(plan: Plan, local_pool, remote_pools, src_block_tables, seq_lens,
                            dst_block_tables, stream=None, check: bool = True) -> int:
    m = max(amoeba_plan_merge_factor(plan), 1)
    rc = lib().amoeba_merge_kv_inplace(plan.handle, _ptr(local_pool), _ptr_array(remote_pools, m),
                                       _ptr_array(src_block_tables, m), _ptr_array(seq_lens, m),
                                       _ptr(dst_block_tables), _stream_handle(stream))
    if check and rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return rc


def amoeba_merge_kv_base(plan: Plan, pools, src_block_tables, seq_lens, new_pool,
                         dst_block_tables, local_blocks_bound: int = 0, stream=None,
                         check: bool = True) -> int:
    m = max(plan.dst_tp // max(plan.src_tp, 1), 1)
    rc = lib().amoeba_merge_kv_base(plan.handle, _ptr_array(pools, m),
                                    _ptr_array(src_block_tables, m), _ptr_array(seq_lens, m),
                                    _ptr(new_pool), _ptr(dst_block_tables), local_blocks_bound,
                                    _stream_handle(stream))
    if check and rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return rc


def amoeba_merge_kv_status(plan: Plan, stream=None):
    """Synchronises the stream; returns (status, remote_blocks_per_layer)."""
    total = ctypes.c_int64(0)
    rc = lib().amoeba_merge_kv_status(plan.handle, _stream_handle(stream), ctypes.byref(total))
    return rc, int(total.value)


def amoeba_plan_padded_info(plan: Plan, side: int):
    """(attn, attn_padded, part, part_padded, stride, layer) in bytes for a padded side."""
    out = (ctypes.c_int64 * 6)()
    rc = lib().amoeba_plan_padded_info(plan.handle, side, out)
    if rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return tuple(int(x) for x in out)


def amoeba_plan_expert_info(plan: Plan, side: int):
    """(experts per rank, first expert offset, expert tensor bytes, expert stride) of a
    mixture-of-experts plan's side, in bytes."""
    out = (ctypes.c_int64 * 4)()
    rc = lib().amoeba_plan_expert_info(plan.handle, side, out)
    if rc != OK:
        raise AmoebaError(rc, amoeba_last_error())
    return tuple(int(x) for x in out)


def amoeba_plan_ffn_view(plan: Plan):
    """None, or (source rank, byte offset in a source layer, bytes, source layer bytes) when
    the target's FFN partitions are a zero-copy range of a source rank's padded buffer."""
    out = (ctypes.c_int64 * 4)()
    if not lib().amoeba_plan_ffn_view(plan.handle, out):
        return None
    return tuple(int(x) for x in out)
