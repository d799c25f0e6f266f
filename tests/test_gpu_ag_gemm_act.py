"""GPU parity of tl_ag_gemm_act_mul (AllGather + GEMM with the MLP layer's activation folded into the epilogue)
against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up

pytestmark = pytest.mark.gpu
ACTS = {"silu": tl.TL_ACT_SILU_MUL, "gelu": tl.TL_ACT_GELU_MUL}


def run_gated(w, rank, C, mode, act, epochs=1, in_place=False, **cfg):
    M, F, K, R = w["M"], w["F"], w["K"], w["world"]
    ctx = make_ctx(world_size=R, rank=rank, channels_per_rank=C, comm_mode=mode, **cfg)
    dims = [M, 2 * F, K]
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, dims)
    info = tl.tl_resolve(ctx, tl.TL_OP_AG_GEMM, dims)
    gathered = poison((M, K))
    ms = M // R
    shards = [up(s) for s in w["a_shards"]]
    if in_place:
        gathered[rank * ms:(rank + 1) * ms] = shards[rank]
        shards[rank] = gathered[rank * ms:(rank + 1) * ms]
    b = up(tl.pack_gate_up(w["w_gate"], w["w_up"]))
    y = poison((M, F))
    flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    comm = torch.cuda.Stream()
    torch.cuda.synchronize()
    for epoch in range(1, epochs + 1):
        if epoch > 1:
            y.copy_(poison((M, F)))
            torch.cuda.synchronize()
        tl.tl_ag_gemm_act_mul(ctx, shards, gathered, b, y, M, F, K, ACTS[act], flags, epoch, wsp, ws_bytes, torch.cuda.current_stream(), comm)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
    tl.tl_ctx_destroy(ctx)
    return down(gathered), down(y), flags.cpu().numpy(), info


@pytest.mark.parametrize("act", ["silu", "gelu"])
@pytest.mark.parametrize("tile,mode", [((128, 128), "waves"), ((256, 256), "side")])
def test_ragged_shapes_both_activations(act, tile, mode):
    # 4 shards of 280 rows, F = 224 features (2F = 448: a ragged last column tile for both tile widths), K = 320
    w = wl.ag_gemm_gated_inputs(1120, 224, 320, 4, config_id=32)
    m = tl.TL_COMM_WAVES if mode == "waves" else tl.TL_COMM_SIDE_KERNEL
    g, y, flags, info = run_gated(w, 1, 5, m, act, epochs=2, tile_m=tile[0], tile_n=tile[1], comm_workgroups=3)
    assert (info["tile_m"], info["tile_n"]) == tile
    a_ref, _, y_ref = ops.ag_gemm_act_mul(w["a_shards"], w["w_gate"], w["w_up"], act)
    assert np.array_equal(g, a_ref)
    assert_close_bf16(y, y_ref, f"gated {act} tile {tile} {mode}")
    assert not (y == 0x7FC0).any()
    assert flags.tolist() == [2 * info["expected_per_channel"]] * 20


def test_gate_and_up_are_not_swapped():
    """up = 0 gives 0 whatever the gate; gate = 0 gives 0; a large gate passes `up` through (silu(g) -> g)."""
    w = wl.ag_gemm_gated_inputs(256, 64, 128, 2, config_id=33)
    zero = np.zeros_like(w["w_up"])
    _, y, _, _ = run_gated(dict(w, w_up=zero), 0, 1, tl.TL_COMM_WAVES, "silu", comm_workgroups=2)
    assert not (y & 0x7FFF).any()          # +0 or -0 (a negative silu(g) times 0)
    _, y2, _, _ = run_gated(w, 0, 1, tl.TL_COMM_WAVES, "silu", comm_workgroups=2)
    _, _, y_ref = ops.ag_gemm_act_mul(w["a_shards"], w["w_gate"], w["w_up"], "silu")
    _, _, y_swapped = ops.ag_gemm_act_mul(w["a_shards"], w["w_up"], w["w_gate"], "silu")
    assert_close_bf16(y2, y_ref, "gated silu")
    assert ops.rel_frobenius(y2, y_swapped) > 0.1


def test_rejects_what_the_epilogue_cannot_pair():
    ctx = make_ctx(world_size=2, rank=0, comm_mode=tl.TL_COMM_WAVES, tile_m=256, tile_n=224)
    w = wl.ag_gemm_gated_inputs(512, 224, 128, 2, config_id=34)
    shards = [up(s) for s in w["a_shards"]]
    b = up(tl.pack_gate_up(w["w_gate"], w["w_up"]))
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [512, 448, 128])
    flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    args = (shards, poison((512, 128)), b, poison((512, 224)), 512, 224, 128)
    with pytest.raises(tl.TileLinkError) as e:
        tl.tl_ag_gemm_act_mul(ctx, *args, tl.TL_ACT_SILU_MUL, flags, 1, wsp, ws_bytes)      # 7 column blocks per wave: no pairs
    assert e.value.status == tl.TL_ERR_UNSUPPORTED_SHAPE
    tl.tl_ctx_destroy(ctx)
    ctx = make_ctx(world_size=2, rank=0, comm_mode=tl.TL_COMM_WAVES)
    with pytest.raises(tl.TileLinkError) as e:
        tl.tl_ag_gemm_act_mul(ctx, *args, 7, flags, 1, wsp, ws_bytes)                         # unknown activation
    assert e.value.status == tl.TL_ERR_INVALID_ARG
    with pytest.raises(tl.TileLinkError) as e:
        tl.tl_ag_gemm_act_mul(ctx, shards, args[1], b, args[3], 512, 200, 128, tl.TL_ACT_SILU_MUL, flags, 1, wsp, ws_bytes)   # F % 32
    assert e.value.status == tl.TL_ERR_UNSUPPORTED_SHAPE
    torch.cuda.synchronize()
    tl.tl_ctx_destroy(ctx)


def test_full_size_mlp5_share():
    """MLP-5 of the paper's table at TP=8: gate and up of I/8 = 3584 features each (2F = 7168), side-kernel producers,
    local shard in place; sampled output columns (the oracle runs on those features only)."""
    S, H, F, R, rank = 8192, 8192, 3584, 8, 6
    w = wl.ag_gemm_gated_inputs(S, F, H, R, config_id=35)
    g, y, flags, info = run_gated(w, rank, 4, tl.TL_COMM_SIDE_KERNEL, "silu", in_place=True, tile_order=tl.TL_ORDER_OWN_FIRST)
    rng = np.random.Generator(np.random.Philox(350))
    cols = np.array(sorted(set(range(8)) | set(range(F - 8, F)) | set(rng.choice(F, size=256, replace=False).tolist())))
    a_ref, _, y_ref = ops.ag_gemm_act_mul(w["a_shards"], np.ascontiguousarray(w["w_gate"][:, cols]), np.ascontiguousarray(w["w_up"][:, cols]), "silu")
    assert np.array_equal(g, a_ref)
    assert_close_bf16(y[:, cols], y_ref, "MLP-5 gated share")
    assert not (y == 0x7FC0).any()
