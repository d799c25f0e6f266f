"""GPU parity of tl_gemm_rs against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import mapping as omap
from oracle import ops
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up

pytestmark = pytest.mark.gpu

MODES = {"waves": tl.TL_COMM_WAVES, "side": tl.TL_COMM_SIDE_KERNEL, "stream": tl.TL_COMM_STREAM}


def run_gemm_rs(w, mode, epochs=1, **cfg):
    M, N, K, R, rank = w["M"], w["N"], w["K"], w["world"], w["rank"]
    ctx = make_ctx(world_size=R, rank=rank, comm_mode=mode, **cfg)
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
    info = tl.tl_resolve(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
    seg = M // R
    a, b = up(w["a"]), up(w["b"])
    partial = poison((M, N))
    recv = [None if q == rank else up(w["peer_segments"][q]) for q in range(R)]
    push = [None if q == rank else poison((seg, N)) for q in range(R)]
    out = poison((seg, N))
    flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    comm = torch.cuda.Stream()
    torch.cuda.synchronize()   # the zero fills above ran on the default stream; the communication stream does not order after it
    host_a = w["a"]
    for epoch in range(1, epochs + 1):
        if epoch > 1:
            host_a = wl.normal_bf16(host_a.shape, 1.0, 78, epoch)
            a.copy_(up(host_a))
            out.copy_(poison((seg, N)))
        torch.cuda.synchronize()
        tl.tl_gemm_rs(ctx, a, b, partial, [0 if t is None else t for t in recv], [0 if t is None else t for t in push], out,
                      M, N, K, flags, epoch, wsp, ws_bytes, torch.cuda.current_stream(), comm)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
    tl.tl_ctx_destroy(ctx)
    return host_a, down(partial), [None if t is None else down(t) for t in push], down(out), flags.cpu().numpy(), info


def check(w, host_a, partial, push, out, what, direct=False):
    R, rank = w["world"], w["rank"]
    seg = w["M"] // R
    p_ref, _, out_ref = ops.gemm_rs(host_a, w["b"], w["peer_segments"], rank)
    if direct:
        # the GEMM epilogue stored segment q's rows straight into peer q's landing zone; `partial` holds the own segment only
        assert_close_bf16(partial[rank * seg:(rank + 1) * seg], p_ref[rank * seg:(rank + 1) * seg], what + " partial (own segment)")
        for q in range(R):
            if q != rank:
                assert (partial[q * seg:(q + 1) * seg] == 0x7FC0).all(), f"{what}: partial rows of segment {q} were written"
                assert_close_bf16(push[q], p_ref[q * seg:(q + 1) * seg], f"{what}: push to peer {q}")
    else:
        assert_close_bf16(partial, p_ref, what + " partial")
        for q in range(R):
            if q != rank:
                # what was pushed to peer q is exactly this rank's partial rows of segment q
                assert np.array_equal(push[q], partial[q * seg:(q + 1) * seg]), f"{what}: push to peer {q}"
    # the reduction of the GPU's own partial with the peers' rows, recomputed by the oracle: tight check of the reducer
    own = partial[rank * seg:(rank + 1) * seg]
    red = ops.reduce_scatter_segment(own, w["peer_segments"], rank)
    from oracle.bf16 import round_to_bf16, widen
    exact = round_to_bf16(red)
    diff = np.abs(widen(out) - widen(exact))
    assert np.all(diff <= np.abs(widen(exact)) * 2.0 ** -7 + 1e-30), f"{what}: reducer differs by more than one bf16 ulp"
    assert np.mean(out != exact) < 0.02, f"{what}: too many last-bit differences in the reducer"
    return assert_close_bf16(out, out_ref, what + " out")


@pytest.mark.parametrize("direct", [0, 1, 2])
@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("rank", [0, 1])
def test_small(mode, rank, direct):
    w = wl.gemm_rs_inputs(256, 512, 512, 2, rank, config_id=21)
    ha, partial, push, out, flags, info = run_gemm_rs(w, MODES[mode], epochs=3, comm_workgroups=2, rs_direct_push=direct)
    check(w, ha, partial, push, out, f"small {mode} r={rank} direct={direct}", direct=bool(direct))
    n_rt = info["n_comm_tiles"]
    tps = n_rt // 2
    ready, arrived, pushed = flags[:n_rt], flags[n_rt:n_rt + 2 * tps], flags[n_rt + 2 * tps:]
    assert ready.tolist() == [3] * n_rt                          # one GEMM tile per reduce tile here
    other = 1 - rank
    assert arrived[other * tps:(other + 1) * tps].tolist() == [3] * tps and arrived[rank * tps:(rank + 1) * tps].tolist() == [0] * tps
    assert pushed[other * tps:(other + 1) * tps].tolist() == [3] * tps and pushed[rank * tps:(rank + 1) * tps].tolist() == [0] * tps


@pytest.mark.parametrize("direct", [0, 1, 2])
@pytest.mark.parametrize("tile,rt", [((256, 256), (56, 152)), ((256, 224), (140, 456)), ((128, 128), (280, 8)), ((128, 128), (20, 152))])
def test_ragged_and_mismatched_reduce_tiles(tile, rt, direct):
    # 4 segments of 280 rows, N = 456: ragged for every GEMM tile (a 256-row tile straddles two segments, so with
    # direct push its rows go to two different places); reduce tiles smaller and larger than GEMM tiles
    w = wl.gemm_rs_inputs(1120, 456, 192, 4, 1, config_id=22)
    ha, partial, push, out, flags, info = run_gemm_rs(w, tl.TL_COMM_WAVES, epochs=2, tile_m=tile[0], tile_n=tile[1],
                                                      comm_tile_m=rt[0], comm_tile_n=rt[1], comm_workgroups=3, rs_direct_push=direct)
    check(w, ha, partial, push, out, f"ragged tile={tile} reduce={rt} direct={direct}", direct=bool(direct))
    table = omap.rs_tile_table(1120, 456, 4, 1, tile[0], tile[1], rt[0], rt[1])
    assert flags[:len(table)].tolist() == [2 * e[7] for e in table]
    # every reduce tile of another rank's segment is announced to its owner exactly once per call, whether the GEMM tile
    # that fills it alone does so itself (direct push) or the reduce side forwards it; nothing is announced for the own segment
    n_rt, tps = len(table), len(table) // 4
    pushed = flags[n_rt + 4 * tps:n_rt + 8 * tps].reshape(4, tps)
    for q in range(4):
        assert pushed[q].tolist() == [0 if q == 1 else 2] * tps, f"pushed counters of segment {q}"


def test_default_reduce_tile_divides_the_segment():
    """M/R = 224 rows per segment, no reduce tile given: the library picks a row count that divides the segment (112
    under 128-row GEMM tiles) instead of refusing the shape."""
    w = wl.gemm_rs_inputs(1120, 256, 128, 5, 3, config_id=23)
    ha, partial, push, out, flags, info = run_gemm_rs(w, tl.TL_COMM_SIDE_KERNEL, epochs=2, comm_workgroups=3, rs_direct_push=1)
    assert 224 % info["comm_tile_m"] == 0
    check(w, ha, partial, push, out, "default reduce tile, 224-row segments", direct=True)


@pytest.mark.parametrize("rank,order,swz", [(0, tl.TL_ORDER_RING, 1), (7, tl.TL_ORDER_RING, 1), (3, tl.TL_ORDER_NATURAL, 0), (5, tl.TL_ORDER_OWN_FIRST, 1)])
def test_schedule_dump_matches_mapping_oracle(rank, order, swz):
    M, N, K, R = 8192, 8192, 3584, 8
    ctx = make_ctx(world_size=R, rank=rank, tile_order=order, xcd_swizzle=swz, comm_tile_m=128, comm_tile_n=512)
    info = tl.tl_resolve(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
    got = tl.tl_dump_schedule(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
    rot = order != tl.TL_ORDER_NATURAL
    own = order == tl.TL_ORDER_OWN_FIRST
    gemm = omap.gemm_rs_schedule_records(M, N, K, R, rank, info["tile_m"], info["tile_n"], 128, 512, info["compute_workgroups"], rot, bool(swz), info["group_m"], own)
    table = omap.rs_tile_table(M, N, R, rank, info["tile_m"], info["tile_n"], 128, 512)
    order_rs = omap.rs_consumer_order(M, N, R, rank, 128, 512, rot, own)
    want = [v for rec in gemm for v in rec]
    for t in order_rs:
        cm, cn, rlo, rhi, clo, chi, dest, exp = table[t]
        want += [t, cm, cn, rlo, rhi, clo, chi, dest, exp]
    assert got == want
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("mode,order,direct", [("waves", tl.TL_ORDER_RING, 0), ("side", tl.TL_ORDER_OWN_FIRST, 0), ("side", tl.TL_ORDER_OWN_FIRST, 1), ("side", tl.TL_ORDER_OWN_FIRST, 2),
                                               ("waves", tl.TL_ORDER_RING, 2)])
def test_full_size_tp8_share(mode, order, direct):
    """BASELINE configuration 3: A [8192,3584] x B [3584,8192], 7 peers, output [1024,8192]; the side-kernel /
    own-first combination is the launch configuration bench.py times."""
    w = wl.gemm_rs_inputs(8192, 8192, 3584, 8, 0, config_id=3)
    ha, partial, push, out, flags, info = run_gemm_rs(w, MODES[mode], epochs=2, tile_order=order, rs_direct_push=direct)
    rel, mx = check(w, ha, partial, push, out, f"cfg3 {mode} direct={direct}", direct=bool(direct))
    print(f"cfg3 {mode}: tile {info['tile_m']}x{info['tile_n']} rel_fro={rel:.2e} max={mx:.2e}")
