"""GPU parity of the MoE entry points (routing tables, AG+gather+grouped GEMM, grouped GEMM+scatter+top-k reduce+RS)
against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from oracle.bf16 import round_to_bf16, widen
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up

pytestmark = pytest.mark.gpu
MODES = {"waves": tl.TL_COMM_WAVES, "side": tl.TL_COMM_SIDE_KERNEL}
ACTS = {"silu": tl.TL_ACT_SILU_MUL, "gelu": tl.TL_ACT_GELU_MUL}


def route_on_gpu(ctx, logits, T, E, k, tile_m, max_tiles, renorm=True):
    d = dev()
    lg = torch.from_numpy(logits).to(d)
    ids = torch.full((T, k), -1, dtype=torch.int32, device=d)
    w = torch.zeros((T, k), dtype=torch.float32, device=d)
    off = torch.full((E + 1,), -1, dtype=torch.int32, device=d)
    srow = torch.full((T * k,), -1, dtype=torch.int32, device=d)
    tab = torch.full((max_tiles, 8), -7, dtype=torch.int32, device=d)
    nt = torch.zeros(1, dtype=torch.int32, device=d)
    tl.tl_moe_route(ctx, lg, T, E, k, renorm, tile_m, ids, w, off, srow, tab, nt)
    torch.cuda.synchronize()
    return ids, w, off, srow, tab, nt


def check_routing(w_in, R, C, tile_m, got, renorm=True):
    T, E, k = w_in["T"], w_in["E"], w_in["topk"]
    ids, w, off, srow, tab, nt = got
    ids_ref, w_ref = ops.moe_route(w_in["logits"], k, renorm)
    _, off_ref, srow_ref = ops.moe_sort_rows(ids_ref, E)
    tab_ref = ops.moe_tile_tables(off_ref, srow_ref, T, k, R, C, tile_m)
    assert np.array_equal(ids.cpu().numpy(), ids_ref)
    assert np.allclose(w.cpu().numpy(), w_ref, rtol=2e-6, atol=1e-7)
    assert np.array_equal(off.cpu().numpy(), off_ref)
    assert np.array_equal(srow.cpu().numpy(), srow_ref)
    n = int(nt.item())
    assert n == len(tab_ref)
    assert np.array_equal(tab.cpu().numpy()[:n], tab_ref)
    return ids_ref, w_ref, off_ref, srow_ref


@pytest.mark.parametrize("T,E,k,R,C,tile_m,renorm", [(64, 4, 2, 2, 2, 16, True), (256, 8, 3, 4, 1, 128, False), (8192, 32, 2, 8, 4, 256, True), (1000, 5, 5, 5, 2, 128, True),
                                                    (8192, 32, 2, 8, 8, 4, True),      # > 2048 tiles: tables assembled in global memory; 64 channels
                                                    (4096, 64, 8, 4, 2, 64, True)])    # the largest expert count and top-k
def test_route_tables_bit_exact(T, E, k, R, C, tile_m, renorm):
    logits = wl.normal_f32((T, E), 1.0, 41, 0)
    # plant ties: equal logits inside some rows must go to the lower expert index
    logits[::7, 1] = logits[::7, 0]
    if E > 3:
        logits[::5, 3] = logits[::5, 2]
    ctx = make_ctx(world_size=R, rank=0, channels_per_rank=C)
    got = route_on_gpu(ctx, logits, T, E, k, tile_m, -(-T * k // tile_m) + E, renorm)
    check_routing(dict(T=T, E=E, topk=k, logits=logits), R, C, tile_m, got, renorm)
    tl.tl_ctx_destroy(ctx)


def run_part1(w, rank, C, mode, epochs=1, act=None, **cfg):
    """`act` "silu" / "gelu": the gated part 1 (W1 = gate, w1_up = up, I features each, packed per expert)."""
    T, H, I, E, k, R = w["T"], w["H"], w["I"], w["E"], w["topk"], w["world"]
    ctx = make_ctx(world_size=R, rank=rank, channels_per_rank=C, comm_mode=mode, **cfg)
    q = tl.tl_moe_query(ctx, tl.TL_OP_MOE_AG_GATHER_GEMM, T, H, 2 * I if act else I, E, k)
    got = route_on_gpu(ctx, w["logits"], T, E, k, q["tile_m"], q["max_row_tiles"])
    ids_ref, w_ref, off_ref, srow_ref = check_routing(w, R, C, q["tile_m"], got)
    ids, tw, off, srow, tab, nt = got
    shards = [up(s) for s in w["x_shards"]]
    xg = poison((T, H))
    if act and I % 32:
        w1 = poison((E * H, 2 * I))      # no packed layout exists: the call has to refuse it
    elif act:
        w1 = up(tl.pack_gate_up(w["w1"].reshape(E * H, I), w["w1_up"].reshape(E * H, I)))
    else:
        w1 = up(w["w1"].reshape(E * H, I))
    y1 = poison((T * k, I))
    flags = torch.zeros(q["n_flags"], dtype=torch.int32, device=dev())
    wsp = torch.zeros(q["ws_bytes"] // 4, dtype=torch.int32, device=dev())
    comm = torch.cuda.Stream()
    torch.cuda.synchronize()   # the zero fills above ran on the default stream; the communication stream does not order after it
    host_shards = [s.copy() for s in w["x_shards"]]
    for epoch in range(1, epochs + 1):
        if epoch > 1:
            for r_ in range(R):
                host_shards[r_] = wl.normal_bf16(host_shards[r_].shape, 1.0, 79, epoch, r_)
                shards[r_].copy_(up(host_shards[r_]))
            y1.copy_(poison((T * k, I)))
        torch.cuda.synchronize()
        tail = (flags, epoch, wsp, q["ws_bytes"], torch.cuda.current_stream(), comm)
        if act:
            tl.tl_moe_ag_gather_gemm_act_mul(ctx, shards, xg, w1, srow, tab, nt, y1, T, H, I, E, k, ACTS[act], *tail)
        else:
            tl.tl_moe_ag_gather_gemm(ctx, shards, xg, w1, srow, tab, nt, y1, T, H, I, E, k, *tail)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
    if act:
        x_ref, _, y_ref = ops.moe_ag_gather_gemm_act_mul(host_shards, w["w1"], w["w1_up"], srow_ref, off_ref, k, act)
    else:
        x_ref, _, y_ref = ops.moe_ag_gather_gemm(host_shards, w["w1"], srow_ref, off_ref, k)
    if mode != tl.TL_COMM_NONE:
        assert np.array_equal(down(xg), x_ref)
        assert flags.cpu().numpy().tolist() == [epochs * q["expected_per_channel"]] * (R * C)
    tl.tl_ctx_destroy(ctx)
    return assert_close_bf16(down(y1), y_ref, "MoE part 1"), q


@pytest.mark.parametrize("mode", list(MODES))
def test_part1_small(mode):
    w = wl.moe_inputs(256, 128, 192, 4, 2, 2, 0, config_id=42)
    run_part1(w, 1, 2, MODES[mode], epochs=2, comm_workgroups=2)


@pytest.mark.parametrize("mode", ["waves", "side"])
def test_part1_simulated_links(mode):
    """Token shards arriving over simulated links (interleaved queue, paced tiles, consumers only wait): same results."""
    w = wl.moe_inputs(512, 128, 192, 4, 2, 4, 1, config_id=44)
    run_part1(w, 1, 2, MODES[mode], epochs=2, comm_workgroups=4, link_gbps=400)


def test_part1_ragged_tiles_and_many_channels():
    # 5 ranks, 5 experts, top-3, I = 320 (ragged for every tile width), explicit 128x128 tile -> short last tiles per expert
    w = wl.moe_inputs(640, 192, 320, 5, 3, 5, 2, config_id=43)
    run_part1(w, 2, 4, tl.TL_COMM_WAVES, epochs=2, comm_workgroups=3, tile_m=128, tile_n=128, comm_tile_m=8, comm_tile_n=64)
    run_part1(w, 2, 4, tl.TL_COMM_SIDE_KERNEL, comm_workgroups=3, tile_m=256, tile_n=224)


@pytest.mark.parametrize("act", ["silu", "gelu"])
@pytest.mark.parametrize("tile,mode", [((128, 128), "waves"), ((256, 256), "side")])
def test_part1_gated_ragged(act, tile, mode):
    """Expert FFN activation folded into the grouped GEMM's epilogue: 5 ranks, 5 experts, top-3, 224 features per half
    (2F = 448: a ragged last column tile for both widths), short last row tiles per expert, two epochs."""
    w = wl.moe_inputs(640, 192, 224, 5, 3, 5, 2, config_id=45)
    (_, _), q = run_part1(w, 2, 4, MODES[mode], epochs=2, act=act, comm_workgroups=3, tile_m=tile[0], tile_n=tile[1])
    assert (q["tile_m"], q["tile_n"]) == tile


def test_part1_gated_rejects_unpaired_tile_and_odd_features():
    w = wl.moe_inputs(256, 128, 224, 4, 2, 2, 0, config_id=46)
    with pytest.raises(tl.TileLinkError) as e:
        run_part1(w, 0, 1, tl.TL_COMM_WAVES, act="silu", comm_workgroups=2, tile_m=256, tile_n=224)
    assert e.value.status == tl.TL_ERR_UNSUPPORTED_SHAPE
    w = wl.moe_inputs(256, 128, 208, 4, 2, 2, 0, config_id=46)          # F % 32 != 0
    with pytest.raises(tl.TileLinkError) as e:
        run_part1(w, 0, 1, tl.TL_COMM_WAVES, act="silu", comm_workgroups=2)
    assert e.value.status == tl.TL_ERR_UNSUPPORTED_SHAPE
    torch.cuda.synchronize()


def test_part2_default_reduce_tile_divides_the_segment():
    """T/R = 192 tokens per rank, no reduce tile given: 96-token reduce tiles instead of a refusal."""
    w = wl.moe_inputs(768, 256, 128, 7, 3, 4, 2, config_id=47)
    q = run_part2(w, tl.TL_COMM_SIDE_KERNEL, epochs=2, rs_direct_push=1, comm_workgroups=4)
    assert 192 % q["tokens_per_reduce_tile"] == 0 and q["tokens_per_reduce_tile"] > 1


def run_part2(w, mode, epochs=1, **cfg):
    T, H, I, E, k, R, rank = w["T"], w["H"], w["I"], w["E"], w["topk"], w["world"], w["rank"]
    ctx = make_ctx(world_size=R, rank=rank, comm_mode=mode, **cfg)
    q = tl.tl_moe_query(ctx, tl.TL_OP_MOE_GEMM_SCATTER_RS, T, H, I, E, k)
    got = route_on_gpu(ctx, w["logits"], T, E, k, q["tile_m"], q["max_row_tiles"])
    ids_ref, w_ref, off_ref, srow_ref = check_routing(w, R, 1, q["tile_m"], got)
    ids, tw, off, srow, tab, nt = got
    seg = T // R
    x2 = up(w["x2"])
    w2 = up(w["w2"].reshape(E * I, H))
    scatter = poison((T * k, H))
    partial = poison((T, H))
    recv = [0 if q_ == rank else up(w["peer_segments"][q_]) for q_ in range(R)]
    push_t = [None if q_ == rank else poison((seg, H)) for q_ in range(R)]
    out = poison((seg, H))
    flags = torch.zeros(q["n_flags"], dtype=torch.int32, device=dev())
    wsp = torch.zeros(q["ws_bytes"] // 4, dtype=torch.int32, device=dev())
    comm = torch.cuda.Stream()
    torch.cuda.synchronize()   # the zero fills above ran on the default stream; the communication stream does not order after it
    host_x2 = w["x2"]
    for epoch in range(1, epochs + 1):
        if epoch > 1:
            host_x2 = wl.normal_bf16(host_x2.shape, 1.0, 80, epoch)
            x2.copy_(up(host_x2))
            out.copy_(poison((seg, H)))
        torch.cuda.synchronize()
        tl.tl_moe_gemm_scatter_rs(ctx, x2, w2, srow, tab, nt, tw, scatter, partial, recv, [0 if t is None else t for t in push_t], out,
                                  T, H, I, E, k, flags, epoch, wsp, q["ws_bytes"], torch.cuda.current_stream(), comm)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
    tl.tl_ctx_destroy(ctx)
    s_ref, p_ref, _, out_ref = ops.moe_gemm_scatter_rs(host_x2, w["w2"], srow_ref, off_ref, w_ref, w["peer_segments"], rank)
    assert_close_bf16(down(scatter), s_ref, "MoE part 2 scatter")
    if mode == tl.TL_COMM_NONE:
        return q
    pg = down(partial)
    if cfg.get("rs_direct_push"):
        # stage B stored the other segments' token blocks straight into the peers' landing zones: reassemble
        for q_ in range(R):
            if q_ != rank:
                assert (pg[q_ * seg:(q_ + 1) * seg] == 0x7FC0).all(), f"partial rows of segment {q_} were written"
                pg[q_ * seg:(q_ + 1) * seg] = down(push_t[q_])
    assert_close_bf16(pg, p_ref, "MoE part 2 partial")
    # the GPU's own top-k reduce and ReduceScatter, recomputed by the oracle from the GPU's intermediate tensors (tight)
    sc = down(scatter)
    p_exact = round_to_bf16(widen(sc).reshape(T, k, H).sum(axis=1))
    assert np.mean(pg != p_exact) < 0.02 and np.all(np.abs(widen(pg) - widen(p_exact)) <= np.abs(widen(p_exact)) * 2.0 ** -7 + 1e-30)
    for q_ in range(R):
        if q_ != rank:
            assert np.array_equal(down(push_t[q_]), pg[q_ * seg:(q_ + 1) * seg]), f"push to peer {q_}"
    red = round_to_bf16(ops.reduce_scatter_segment(pg[rank * seg:(rank + 1) * seg], w["peer_segments"], rank))
    og = down(out)
    assert np.mean(og != red) < 0.02 and np.all(np.abs(widen(og) - widen(red)) <= np.abs(widen(red)) * 2.0 ** -7 + 1e-30)
    assert_close_bf16(og, out_ref, "MoE part 2 out")
    # counters: every (token block, column block) received Tt*topk rows per call; every reduce tile one notification
    ntb, nbn, Tt = T // q["tokens_per_reduce_tile"], q["col_blocks"], q["tokens_per_reduce_tile"]
    f = flags.cpu().numpy()
    assert f[:ntb * nbn].tolist() == [epochs * Tt * k] * (ntb * nbn)
    assert f[ntb * nbn:2 * ntb * nbn].tolist() == [epochs] * (ntb * nbn)
    # ... then the peers' arrivals (simulated: all but the own segment's row) and this rank's announcements to the owners:
    # once per call for every reduce tile of another segment, by stage B itself with direct push, else by stage C
    tps = (ntb // R) * nbn
    arrived = f[2 * ntb * nbn:2 * ntb * nbn + R * tps].reshape(R, tps)
    pushed = f[2 * ntb * nbn + R * tps:2 * ntb * nbn + 2 * R * tps].reshape(R, tps)
    for q_ in range(R):
        assert arrived[q_].tolist() == [0 if q_ == rank else epochs] * tps and pushed[q_].tolist() == [0 if q_ == rank else epochs] * tps
    return q


@pytest.mark.parametrize("direct", [0, 1])
@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("rank", [0, 1])
def test_part2_small(mode, rank, direct):
    w = wl.moe_inputs(256, 256, 128, 4, 2, 2, rank, config_id=44)
    run_part2(w, MODES[mode], epochs=2, comm_workgroups=4, rs_direct_push=direct)


def test_part2_gemm_stage_only_and_other_shapes():
    w = wl.moe_inputs(640, 512, 192, 5, 3, 5, 3, config_id=45)
    run_part2(w, tl.TL_COMM_NONE)
    run_part2(w, tl.TL_COMM_WAVES, epochs=2, comm_workgroups=5, comm_tile_m=64, tile_m=256, tile_n=256)
    run_part2(w, tl.TL_COMM_SIDE_KERNEL, comm_workgroups=6, tile_m=128, tile_n=128, tile_order=tl.TL_ORDER_OWN_FIRST)
    run_part2(w, tl.TL_COMM_SIDE_KERNEL, comm_workgroups=6, tile_m=256, tile_n=256, tile_order=tl.TL_ORDER_OWN_FIRST, rs_direct_push=1)


@pytest.mark.parametrize("mode", ["side"])
def test_full_size_tp8_share(mode):
    """BASELINE configuration 4: 8192 tokens, hidden 4096, 32 experts top-2, per-rank expert FFN slice 4096 -> 1792."""
    w = wl.moe_inputs(8192, 4096, 1792, 32, 2, 8, 0, config_id=4)
    (rel, mx), q1 = run_part1(w, 0, 4, MODES[mode])
    print(f"cfg4 part1 {mode}: tile {q1['tile_m']}x{q1['tile_n']} rel_fro={rel:.2e} max={mx:.2e}")
    q2 = run_part2(w, MODES[mode], tile_order=tl.TL_ORDER_OWN_FIRST)
    print(f"cfg4 part2 {mode}: tile {q2['tile_m']}x{q2['tile_n']}")
    run_part2(w, MODES[mode], tile_order=tl.TL_ORDER_OWN_FIRST, rs_direct_push=1)
