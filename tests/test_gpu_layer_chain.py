"""GPU parity of whole layers (paper, evaluation: "MLP Layer" and "MoE Layer"): the first half's GPU output, left in
device memory, is the second half's input; the final shard is compared with the oracle composing the same two
functions on the ORACLE's own intermediate tensor.  The intermediate differs from the oracle's by bf16 rounding flips,
which the tolerance of the final comparison has to absorb like any other rounding."""
import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up
from tests.test_gpu_moe import check_routing, route_on_gpu

pytestmark = pytest.mark.gpu


def run_mlp_layer(S, H, F, R, rank, act, cols=None, **cfg):
    """AllGather + GEMM over gate|up weights with the activation in the epilogue, then GEMM + ReduceScatter on its
    output.  Returns (out bits of the GPU, out bits of the oracle, y GPU, y oracle); with `cols` the second half of the
    oracle runs on those output columns only (the GPU always computes everything)."""
    w1 = wl.ag_gemm_gated_inputs(S, F, H, R, config_id=120)
    w2 = wl.gemm_rs_inputs(S, H, F, R, rank, config_id=121)      # only its B (the down projection) and the peers' rows are used
    seg = S // R
    ctx1 = make_ctx(world_size=R, rank=rank, channels_per_rank=2, **cfg)
    ctx2 = make_ctx(world_size=R, rank=rank, rs_direct_push=1, **cfg)
    ws1, nf1 = tl.tl_query_workspace(ctx1, tl.TL_OP_AG_GEMM, [S, 2 * F, H])
    ws2, nf2 = tl.tl_query_workspace(ctx2, tl.TL_OP_GEMM_RS, [S, H, F])
    shards = [up(s) for s in w1["a_shards"]]
    gathered, y = poison((S, H)), poison((S, F))
    b_gu, b_down = up(tl.pack_gate_up(w1["w_gate"], w1["w_up"])), up(w2["b"])
    partial, out = poison((S, H)), poison((seg, H))
    recv = [0 if q == rank else up(w2["peer_segments"][q]) for q in range(R)]
    push = [0 if q == rank else poison((seg, H)) for q in range(R)]
    f1, f2 = torch.zeros(nf1, dtype=torch.int32, device=dev()), torch.zeros(nf2, dtype=torch.int32, device=dev())
    p1, p2 = torch.zeros(ws1 // 4, dtype=torch.int32, device=dev()), torch.zeros(ws2 // 4, dtype=torch.int32, device=dev())
    cs, ms = torch.cuda.current_stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    tl.tl_ag_gemm_act_mul(ctx1, shards, gathered, b_gu, y, S, F, H, tl.TL_ACT_SILU_MUL if act == "silu" else tl.TL_ACT_GELU_MUL, f1, 1, p1, ws1, cs, ms)
    ms.wait_stream(cs)          # the reduce side of the second half may not run ahead into the first half
    tl.tl_gemm_rs(ctx2, y, b_down, partial, recv, push, out, S, H, F, f2, 1, p2, ws2, cs, ms)
    torch.cuda.synchronize()
    tl.tl_check_status(ctx1, p1)
    tl.tl_check_status(ctx2, p2)
    tl.tl_ctx_destroy(ctx1)
    tl.tl_ctx_destroy(ctx2)
    _, _, y_ref = ops.ag_gemm_act_mul(w1["a_shards"], w1["w_gate"], w1["w_up"], act)
    if cols is None:
        cols = np.arange(H)
    peers = [None if p is None else np.ascontiguousarray(p[:, cols]) for p in w2["peer_segments"]]
    p_ref, _, out_ref = ops.gemm_rs(y_ref, np.ascontiguousarray(w2["b"][:, cols]), peers, rank)
    got_push = {q: down(push[q])[:, cols] for q in range(R) if q != rank}
    return down(out)[:, cols], out_ref, down(y), y_ref, got_push, p_ref


@pytest.mark.parametrize("act,mode,rank", [("silu", "side", 1), ("gelu", "waves", 3)])
def test_mlp_layer_mid_size(act, mode, rank):
    # 4 ranks, 1120 tokens (ragged row tiles), hidden 512, 448 features per rank (K of the second half = 14 steps of 32)
    m = tl.TL_COMM_SIDE_KERNEL if mode == "side" else tl.TL_COMM_WAVES
    out, out_ref, y, y_ref, push, p_ref = run_mlp_layer(1120, 512, 448, 4, rank, act, comm_mode=m, comm_workgroups=4, tile_order=tl.TL_ORDER_OWN_FIRST)
    assert_close_bf16(y, y_ref, f"MLP layer {act}: activation output")
    assert_close_bf16(out, out_ref, f"MLP layer {act} {mode}: reduced shard")
    for q, t in push.items():
        assert_close_bf16(t, p_ref[q * 280:(q + 1) * 280], f"MLP layer {act}: rows pushed to rank {q}")


def test_mlp_layer_mlp5_share():
    """MLP-5 of the paper's table at TP=8, rank 0, the bindings bench.py times: S=8192, H=8192, 3584 features per rank.
    The oracle computes the whole intermediate and the second half on sampled output columns."""
    S, H, F, R = 8192, 8192, 3584, 8
    rng = np.random.Generator(np.random.Philox(1200))
    cols = np.array(sorted(set(range(8)) | set(range(H - 8, H)) | set(rng.choice(H, size=256, replace=False).tolist())))
    out, out_ref, y, y_ref, push, p_ref = run_mlp_layer(S, H, F, R, 0, "silu", cols=cols, comm_mode=tl.TL_COMM_SIDE_KERNEL,
                                                        tile_order=tl.TL_ORDER_OWN_FIRST)
    assert_close_bf16(y, y_ref, "MLP-5 layer: activation output")
    assert_close_bf16(out, out_ref, "MLP-5 layer: reduced shard")
    seg = S // R
    for q, t in push.items():
        assert_close_bf16(t, p_ref[q * seg:(q + 1) * seg], f"MLP-5 layer: rows pushed to rank {q}")


def run_moe_layer(T, H, F, E, k, R, rank, act, config_id, **cfg):
    """AllGather + gather + grouped GEMM over gate|up expert weights with the activation in the epilogue, then grouped
    GEMM + scatter + top-k reduce + ReduceScatter on its output."""
    w = wl.moe_inputs(T, H, F, E, k, R, rank, config_id=config_id)
    ctx1 = make_ctx(world_size=R, rank=rank, channels_per_rank=2, **cfg)
    ctx2 = make_ctx(world_size=R, rank=rank, rs_direct_push=1, **cfg)
    q1 = tl.tl_moe_query(ctx1, tl.TL_OP_MOE_AG_GATHER_GEMM, T, H, 2 * F, E, k)
    q2 = tl.tl_moe_query(ctx2, tl.TL_OP_MOE_GEMM_SCATTER_RS, T, H, F, E, k)
    r1 = route_on_gpu(ctx1, w["logits"], T, E, k, q1["tile_m"], q1["max_row_tiles"])
    r2 = route_on_gpu(ctx2, w["logits"], T, E, k, q2["tile_m"], q2["max_row_tiles"])
    ids_ref, w_ref, off_ref, srow_ref = check_routing(w, R, 2, q1["tile_m"], r1)
    check_routing(w, R, 1, q2["tile_m"], r2)
    seg = T // R
    shards = [up(s) for s in w["x_shards"]]
    xg, y1 = poison((T, H)), poison((T * k, F))
    w1 = up(tl.pack_gate_up(w["w1"].reshape(E * H, F), w["w1_up"].reshape(E * H, F)))
    w2 = up(w["w2"].reshape(E * F, H))
    scatter, partial, out = poison((T * k, H)), poison((T, H)), poison((seg, H))
    recv = [0 if q == rank else up(w["peer_segments"][q]) for q in range(R)]
    push = [0 if q == rank else poison((seg, H)) for q in range(R)]
    f1, f2 = torch.zeros(q1["n_flags"], dtype=torch.int32, device=dev()), torch.zeros(q2["n_flags"], dtype=torch.int32, device=dev())
    p1, p2 = torch.zeros(q1["ws_bytes"] // 4, dtype=torch.int32, device=dev()), torch.zeros(q2["ws_bytes"] // 4, dtype=torch.int32, device=dev())
    cs, ms = torch.cuda.current_stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    tl.tl_moe_ag_gather_gemm_act_mul(ctx1, shards, xg, w1, r1[3], r1[4], r1[5], y1, T, H, F, E, k, tl.TL_ACT_SILU_MUL if act == "silu" else tl.TL_ACT_GELU_MUL,
                                     f1, 1, p1, q1["ws_bytes"], cs, ms)
    ms.wait_stream(cs)
    tl.tl_moe_gemm_scatter_rs(ctx2, y1, w2, r2[3], r2[4], r2[5], r2[1], scatter, partial, recv, push, out, T, H, F, E, k, f2, 1, p2, q2["ws_bytes"], cs, ms)
    torch.cuda.synchronize()
    tl.tl_check_status(ctx1, p1)
    tl.tl_check_status(ctx2, p2)
    tl.tl_ctx_destroy(ctx1)
    tl.tl_ctx_destroy(ctx2)
    _, _, y_ref = ops.moe_ag_gather_gemm_act_mul(w["x_shards"], w["w1"], w["w1_up"], srow_ref, off_ref, k, act)
    s_ref, p_ref, _, out_ref = ops.moe_gemm_scatter_rs(y_ref, w["w2"], srow_ref, off_ref, w_ref, w["peer_segments"], rank)
    assert_close_bf16(down(y1), y_ref, "MoE layer: activation output")
    assert_close_bf16(down(scatter), s_ref, "MoE layer: scattered rows")
    for q in range(R):
        if q != rank:
            assert_close_bf16(down(push[q]), p_ref[q * seg:(q + 1) * seg], f"MoE layer: token rows pushed to rank {q}")
    assert_close_bf16(down(out), out_ref, "MoE layer: reduced shard")
    assert not (down(out) == 0x7FC0).any()


@pytest.mark.parametrize("act,mode", [("silu", "side"), ("gelu", "waves")])
def test_moe_layer_mid_size(act, mode):
    m = tl.TL_COMM_SIDE_KERNEL if mode == "side" else tl.TL_COMM_WAVES
    run_moe_layer(1024, 512, 192, 8, 2, 4, 2, act, 122, comm_mode=m, comm_workgroups=4, tile_order=tl.TL_ORDER_OWN_FIRST)


def test_moe_layer_config4_share():
    """Configuration 4 (8192 tokens, hidden 4096, 32 experts top-2, 1792 features per rank), rank 0, side kernels."""
    run_moe_layer(8192, 4096, 1792, 32, 2, 8, 0, "silu", 4, comm_mode=tl.TL_COMM_SIDE_KERNEL, tile_order=tl.TL_ORDER_OWN_FIRST)
