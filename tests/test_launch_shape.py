"""Launch geometry (host only): HIP refuses a launch whose grid.x * lanes exceeds 2^32 - 1
work-items, so the launchers clamp the grid and the kernels stride over the rest.  The
geometry comes from amoeba_plan_launch_shape(), which runs the launchers' own arithmetic."""
import pytest

from paper_2509_19729_amd import binding as ab
from paper_2509_19729_amd import workloads as wl

LIMIT = 2 ** 32 - 1


def shape_for(name, **kw):
    w = wl.WORKLOADS[name]
    base = dict(n_layers=w.n_layers, hidden=w.hidden, n_q_heads=w.n_q_heads,
                n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, ffn_dim=w.ffn_dim)
    base.update(kw)
    return ab.ModelShape(**base)


def check(gx, gy, lanes, items, xcd_order=True):
    assert gx >= 1 and gx * lanes <= LIMIT
    assert gx <= max(items, 1)
    if gx < items and xcd_order:         # clamped: whole XCD rounds, so a stride keeps its XCD
        assert gx % 8 == 0 or gx == items


def test_weight_grid_is_one_workgroup_per_tile_until_the_work_item_limit():
    plan = ab.amoeba_plan(shape_for("llama7b"), 4, 2, 1)
    gx, gy, lanes, items = ab.amoeba_plan_launch_shape(plan, ab.KERNEL_WEIGHTS, 16)
    assert lanes == 64 and gy == 1 and gx == items
    assert items * 1024 == ab.amoeba_plan_shard_bytes(plan, 1)   # 1 KiB tiles, no ragged tail here
    # a 70B-shaped TP2 -> TP1 merge of 41 layers: a 65 GiB target shard has more 1 KiB tiles
    # than one grid dimension has room for at 64 lanes
    plan = ab.amoeba_plan(shape_for("gqa70b", n_layers=41), 2, 1, 0)
    nbytes = ab.amoeba_plan_shard_bytes(plan, 1)
    assert nbytes > 64 << 30
    gx, gy, lanes, items = ab.amoeba_plan_launch_shape(plan, ab.KERNEL_WEIGHTS, 16)
    assert lanes == 64 and items * 1024 >= nbytes and items > LIMIT // 64
    assert gx == (LIMIT // 64) // 8 * 8
    check(gx, gy, lanes, items)
    # 4-byte aligned buffers: 256 lanes of 4 bytes, 1 KiB tiles, 13B target shard
    plan = ab.amoeba_plan(shape_for("llama13b"), 2, 1, 0)
    gx, gy, lanes, items = ab.amoeba_plan_launch_shape(plan, ab.KERNEL_WEIGHTS, 4)
    assert lanes == 256 and items > 2 ** 24 and gx == (LIMIT // 256) // 8 * 8
    check(gx, gy, lanes, items)
    # a sweep's grid override is honoured below the limit
    ab.amoeba_plan_tune(plan, ab.TUNE_W_GRID, 4096)
    assert ab.amoeba_plan_launch_shape(plan, ab.KERNEL_WEIGHTS, 16)[0] == 4096


@pytest.mark.parametrize("kv_layers,bound,align", [(1, 0, 16), (1, 0, 2), (4, 0, 16), (80, 0, 16),
                                                    (1, 5000, 16), (2, 10 ** 6, 16)])
def test_kv_grid_stays_inside_the_work_item_limit(kv_layers, bound, align):
    # a large pool of 320 KiB blocks (13B shape at TP1): up to 2^26 tiles per layer
    s = shape_for("llama13b", kv_layers=kv_layers, num_seqs=128, max_blocks_per_seq=256,
                  src_pool_blocks=400000, dst_pool_blocks=400000, kv_blocks_bound=bound)
    plan = ab.amoeba_plan(s, 2, 1, 0)
    gx, gy, lanes, items = ab.amoeba_plan_launch_shape(plan, ab.KERNEL_KV_REGROUP, align)
    assert gy == kv_layers
    assert lanes == (64 if bound and align == 16 else 256)
    check(gx, gy, lanes, items)
    tiles_per_block = items // 400000
    up8 = lambda n: -(-n // 8) * 8
    if bound:
        assert gx == min(up8(bound * tiles_per_block), (LIMIT // lanes) // 8 * 8)
    else:   # the pool's capacity, at most 2^27 workgroups over all layers, at most the limit
        assert gx == min(items, up8(max(2 ** 16, 2 ** 27 // kv_layers)), (LIMIT // 256) // 8 * 8)
        if kv_layers == 1:
            assert gx == (LIMIT // 256) // 8 * 8      # 2^27 workgroups of 256 lanes do not fit


def test_small_tables_take_single_wavefront_workgroups():
    s = shape_for("tiny", kv_layers=2, num_seqs=4, max_blocks_per_seq=32, src_pool_blocks=128,
                  dst_pool_blocks=130)
    plan = ab.amoeba_plan(s, 1, 2, 0)
    gx, gy, lanes, items = ab.amoeba_plan_launch_shape(plan, ab.KERNEL_KV_REGROUP, 16)
    assert (lanes, gy) == (64, 2) and gx == items == 130 * 8     # 8 KiB target blocks
    ab.amoeba_plan_tune(plan, ab.TUNE_KV_SMALL_TABLE, 1)          # three-kernel path, no bound
    assert ab.amoeba_plan_launch_shape(plan, ab.KERNEL_KV_REGROUP, 16)[2] == 256


def test_merge_grid():
    s = shape_for("llama7b", kv_layers=1, num_seqs=16, max_blocks_per_seq=512,
                  src_pool_blocks=300000, dst_pool_blocks=0)
    plan = ab.amoeba_plan(s, 1, 4, 1)
    assert ab.amoeba_plan_merge_factor(plan) == 4
    gx, gy, lanes, items = ab.amoeba_plan_launch_shape(plan, ab.KERNEL_MERGE_COPY, 16)
    assert lanes == 256 and gy == 1 and items == 300000 * 4 * 64   # 64 KiB new blocks
    check(gx, gy, lanes, items, xcd_order=False)                   # the merge copy takes plain order
    assert gx == ((LIMIT // 64) // 8 * 8 + 3) // 4                 # four 1 KiB tiles per workgroup
    with pytest.raises(ab.AmoebaError):
        ab.amoeba_plan_launch_shape(ab.amoeba_plan(shape_for("llama7b"), 4, 2, 1),
                                    ab.KERNEL_MERGE_COPY, 16)
    with pytest.raises(ab.AmoebaError):
        ab.amoeba_plan_launch_shape(plan, 7, 16)
    with pytest.raises(ab.AmoebaError):
        ab.amoeba_plan_launch_shape(plan, ab.KERNEL_WEIGHTS, 3)
