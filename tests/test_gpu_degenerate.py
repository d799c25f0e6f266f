"""Degenerate cases of every operator on the GPU: a single rank (nothing to communicate), experts that receive no
tokens, one expert with top-1 (the MoE halves reduce to the dense operators), the smallest legal shapes."""
import numpy as np
import pytest

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from tests.gpu_util import assert_close_bf16
from tests.test_gpu_ag_gemm import check as check_ag, run_ag_gemm
from tests.test_gpu_attention import check_gathered, run_attention
from tests.test_gpu_gemm_rs import check as check_rs, run_gemm_rs
from tests.test_gpu_moe import run_part1, run_part2

pytestmark = pytest.mark.gpu
MODES = {"waves": tl.TL_COMM_WAVES, "side": tl.TL_COMM_SIDE_KERNEL}


@pytest.mark.parametrize("mode", list(MODES))
def test_single_rank_every_operator(mode):
    """R = 1: the AllGather is a local copy, the ReduceScatter has no peers (out == partial, bit for bit)."""
    m = MODES[mode]
    w = wl.ag_gemm_inputs(256, 256, 128, 1, config_id=101)
    hs, g, c, flags, info = run_ag_gemm(w, 0, 2, m, comm_workgroups=2)
    check_ag(w, hs, g, c, f"R=1 AG+GEMM {mode}")
    w = wl.gemm_rs_inputs(256, 256, 128, 1, 0, config_id=102)
    ha, partial, push, out, flags, info = run_gemm_rs(w, m, comm_workgroups=2, rs_direct_push=1)
    check_rs(w, ha, partial, push, out, f"R=1 GEMM+RS {mode}", direct=True)
    assert np.array_equal(out, partial)
    w = wl.sp_attention_inputs(256, 1, 128, 1, config_id=103)
    res = run_attention(w, 0, True, m)
    _, _, _, o_ref = ops.sp_ag_attention(w["q_shards"][0], w["k_shards"], w["v_shards"], 0, True)
    assert_close_bf16(res["o"], o_ref, f"R=1 attention {mode}")
    check_gathered(w, res, 0, True, 1)


def test_smallest_shapes():
    """One 64-wide K step, 8 output columns, one row per rank."""
    w = wl.ag_gemm_inputs(2, 8, 64, 2, config_id=104)
    hs, g, c, flags, info = run_ag_gemm(w, 1, 1, tl.TL_COMM_WAVES, comm_workgroups=1)
    check_ag(w, hs, g, c, "2x8x64")
    w = wl.gemm_rs_inputs(2, 8, 64, 2, 0, config_id=105)
    ha, partial, push, out, flags, info = run_gemm_rs(w, tl.TL_COMM_SIDE_KERNEL, comm_workgroups=1)
    check_rs(w, ha, partial, push, out, "2x8x64 RS")


@pytest.mark.parametrize("direct", [0, 1])
def test_moe_with_empty_experts(direct):
    """Experts 1, 4 and 7 of 8 get no token at all (their logits are far below the others): no tiles for them, the
    offsets of their neighbours coincide, and both halves still match the oracle."""
    w = wl.moe_inputs(512, 128, 128, 8, 2, 2, 1, config_id=106)
    w["logits"][:, [1, 4, 7]] = -1e9
    ids, _ = ops.moe_route(w["logits"], 2, True)
    assert not np.isin(ids, [1, 4, 7]).any()
    run_part1(w, 1, 2, tl.TL_COMM_WAVES, comm_workgroups=2)
    run_part2(w, tl.TL_COMM_SIDE_KERNEL, comm_workgroups=4, rs_direct_push=direct)


def test_moe_one_expert_top1_is_the_dense_operator():
    """E = 1, k = 1: every token goes to the only expert with weight 1, sorted order = token order; part 1 is AG+GEMM
    with W1[0], part 2 is GEMM+RS with W2[0] (checked against the dense oracles, not only the MoE one)."""
    T, H, I, R, rank = 512, 256, 128, 2, 0
    w = wl.moe_inputs(T, H, I, 1, 1, R, rank, config_id=107)
    run_part1(w, rank, 1, tl.TL_COMM_SIDE_KERNEL, comm_workgroups=2)
    run_part2(w, tl.TL_COMM_WAVES, comm_workgroups=4)
    # the MoE oracle itself against the dense one on the same data
    ids, tw = ops.moe_route(w["logits"], 1, True)
    _, off, srow = ops.moe_sort_rows(ids, 1)
    assert np.array_equal(srow, np.arange(T)) and np.all(tw == 1.0)
    _, _, y_moe = ops.moe_ag_gather_gemm(w["x_shards"], w["w1"], srow, off, 1)
    _, _, y_dense = ops.ag_gemm(w["x_shards"], w["w1"][0])
    assert np.array_equal(y_moe, y_dense)
    _, _, _, out_moe = ops.moe_gemm_scatter_rs(w["x2"], w["w2"], srow, off, tw, w["peer_segments"], rank)
    _, _, out_dense = ops.gemm_rs(w["x2"], w["w2"][0], w["peer_segments"], rank)
    assert np.array_equal(out_moe, out_dense)


def test_query_workspace_covers_every_operator():
    """tl_query_workspace agrees with the operator-specific queries for the MoE halves and attention."""
    from tests.gpu_util import make_ctx
    ctx = make_ctx(world_size=8, rank=3, channels_per_rank=2, comm_mode=tl.TL_COMM_SIDE_KERNEL)
    for op in (tl.TL_OP_MOE_AG_GATHER_GEMM, tl.TL_OP_MOE_GEMM_SCATTER_RS):
        q = tl.tl_moe_query(ctx, op, 8192, 4096, 1792, 32, 2)
        assert tl.tl_query_workspace(ctx, op, [8192, 4096, 1792, 32, 2]) == (q["ws_bytes"], q["n_flags"])
    a = tl.tl_attn_query(ctx, 32768, 32, 128, True)
    assert tl.tl_query_workspace(ctx, tl.TL_OP_SP_AG_ATTENTION, [32768, 32, 128]) == (a["ws_bytes"], a["n_flags"])
    with pytest.raises(tl.TileLinkError):
        tl.tl_query_workspace(ctx, 17, [1, 2, 3])
    tl.tl_ctx_destroy(ctx)
