"""GPU parity of tl_ag_gemm against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import mapping as omap
from oracle import ops
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up

pytestmark = pytest.mark.gpu

MODES = {"waves": tl.TL_COMM_WAVES, "stream": tl.TL_COMM_STREAM, "side": tl.TL_COMM_SIDE_KERNEL, "copy_engine": tl.TL_COMM_COPY_ENGINE}


def run_ag_gemm(w, rank, C, mode, epochs=1, in_place=False, **cfg):
    """Runs `epochs` calls; between calls the shards are replaced with fresh data so that stale
    cache lines of the previous call would show.  Returns the last call's device results."""
    M, N, K, R = w["M"], w["N"], w["K"], w["world"]
    ctx = make_ctx(world_size=R, rank=rank, channels_per_rank=C, comm_mode=mode, **cfg)
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    info = tl.tl_resolve(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    gathered = poison((M, K))
    ms = M // R
    shards = [up(s) for s in w["a_shards"]]
    if in_place:
        gathered[rank * ms:(rank + 1) * ms] = shards[rank]
        shards[rank] = gathered[rank * ms:(rank + 1) * ms]
    b = up(w["b"])
    c = poison((M, N))
    flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    comm = torch.cuda.Stream()
    torch.cuda.synchronize()   # the zero fills above ran on the default stream; the communication stream does not order after it
    host_shards = [s.copy() for s in w["a_shards"]]
    for epoch in range(1, epochs + 1):
        if epoch > 1:
            # new data in every shard, same buffers
            for q in range(R):
                host_shards[q] = wl.normal_bf16(host_shards[q].shape, 1.0, 77, epoch, q)
                shards[q].copy_(up(host_shards[q]))
            c.copy_(poison((M, N)))
        torch.cuda.synchronize()
        tl.tl_ag_gemm(ctx, shards, gathered, b, c, M, N, K, flags, epoch, wsp, ws_bytes, torch.cuda.current_stream(), comm)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
    tl.tl_ctx_destroy(ctx)
    return host_shards, down(gathered), down(c), flags.cpu().numpy(), info


def check(w, host_shards, gathered, c, what):
    a_ref, _, c_ref = ops.ag_gemm(host_shards, w["b"])
    assert np.array_equal(gathered, a_ref), f"{what}: gathered A is not the concatenation of the shards"
    return assert_close_bf16(c, c_ref, what)


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("rank,C", [(0, 1), (1, 2), (0, 2)])
def test_small_config_all_modes(mode, rank, C):
    w = wl.ag_gemm_inputs(256, 512, 512, 2, config_id=1, a_dist="uniform")
    hs, g, c, flags, info = run_ag_gemm(w, rank, C, MODES[mode], epochs=3, comm_workgroups=2)
    check(w, hs, g, c, f"cfg1 {mode} rank={rank} C={C}")
    expected = info["expected_per_channel"] if mode not in ("stream", "copy_engine") else 1
    assert flags.tolist() == [3 * expected] * (2 * C)


@pytest.mark.parametrize("tile", [(256, 256), (256, 224), (128, 128)])
def test_ragged_edges_every_tile_shape(tile):
    # M = 4 shards of 280 rows (not a multiple of any tile height), N = 456 (not a multiple of 128/224/256)
    w = wl.ag_gemm_inputs(1120, 456, 320, 4, config_id=11)
    hs, g, c, flags, info = run_ag_gemm(w, 2, 5, tl.TL_COMM_WAVES, epochs=2, tile_m=tile[0], tile_n=tile[1], comm_workgroups=3, comm_tile_m=8, comm_tile_n=64)
    assert (info["tile_m"], info["tile_n"]) == tile
    check(w, hs, g, c, f"ragged tile={tile}")
    assert flags.tolist() == [2 * (56 // 8) * (320 // 64)] * 20


@pytest.mark.parametrize("mode", ["waves", "side"])
def test_local_shard_in_place(mode):
    w = wl.ag_gemm_inputs(1024, 512, 256, 4, config_id=12)
    hs, g, c, flags, info = run_ag_gemm(w, 3, 1, MODES[mode], in_place=True, comm_workgroups=4)
    check(w, hs, g, c, "in place")


def test_no_comm_mode_uses_pregathered_data():
    w = wl.ag_gemm_inputs(512, 256, 128, 2, config_id=13)
    M, N, K = 512, 256, 128
    ctx = make_ctx(world_size=2, rank=0, comm_mode=tl.TL_COMM_NONE)
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    a_ref, _, c_ref = ops.ag_gemm(w["a_shards"], w["b"])
    gathered = up(a_ref)
    shards = [up(s) for s in w["a_shards"]]
    c = poison((M, N))
    flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    tl.tl_ag_gemm(ctx, shards, gathered, up(w["b"]), c, M, N, K, flags, 1, wsp, ws_bytes)
    torch.cuda.synchronize()
    assert_close_bf16(down(c), c_ref, "no-comm")
    assert flags.cpu().numpy().tolist() == [0, 0]
    tl.tl_ctx_destroy(ctx)


def test_exact_small_integers_bit_exact():
    # integer-valued inputs: every partial sum is exact in fp32, so the GPU must match bit for bit
    g = np.random.default_rng(5)
    from oracle.bf16 import round_to_bf16
    R, M, N, K = 2, 256, 256, 128
    shards = [round_to_bf16(g.integers(-3, 4, size=(M // R, K)).astype(np.float64)) for _ in range(R)]
    b = round_to_bf16(g.integers(-2, 3, size=(K, N)).astype(np.float64))
    w = dict(a_shards=shards, b=b, M=M, N=N, K=K, world=R)
    hs, gathered, c, _, _ = run_ag_gemm(w, 1, 1, tl.TL_COMM_WAVES, comm_workgroups=2)
    _, _, c_ref = ops.ag_gemm(shards, b)
    assert np.array_equal(c, c_ref)


def test_withheld_flag_times_out_instead_of_hanging():
    w = wl.ag_gemm_inputs(256, 128, 64, 2, config_id=14)
    M, N, K = 256, 128, 64
    ctx = make_ctx(world_size=2, rank=0, comm_mode=tl.TL_COMM_EXTERNAL, spin_timeout_us=20_000)
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    shards = [up(s) for s in w["a_shards"]]
    gathered = up(np.concatenate(w["a_shards"]))
    c = poison((M, N))
    flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    expected = tl.tl_resolve(ctx, tl.TL_OP_AG_GEMM, [M, N, K])["expected_per_channel"]
    flags[0] = expected           # rank 0's channel is ready, rank 1's is never raised
    tl.tl_ag_gemm(ctx, shards, gathered, up(w["b"]), c, M, N, K, flags, 1, wsp, ws_bytes)
    torch.cuda.synchronize()
    with pytest.raises(tl.TileLinkError) as e:
        tl.tl_check_status(ctx, wsp)
    assert e.value.status == tl.TL_ERR_TIMEOUT
    # with both flags raised the same call completes and is correct
    flags[1] = expected
    tl.tl_ag_gemm(ctx, shards, gathered, up(w["b"]), c, M, N, K, flags, 1, wsp, ws_bytes)
    torch.cuda.synchronize()
    tl.tl_check_status(ctx, wsp)
    _, _, c_ref = ops.ag_gemm(w["a_shards"], w["b"])
    assert_close_bf16(down(c), c_ref, "external flags")
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("rank,order,swz,gm", [(0, tl.TL_ORDER_RING, 1, 0), (5, tl.TL_ORDER_RING, 1, 8), (3, tl.TL_ORDER_NATURAL, 0, 1), (2, tl.TL_ORDER_RING, 0, 3)])
def test_schedule_dump_matches_mapping_oracle(rank, order, swz, gm):
    M, N, K, R, C = 8192, 3584, 8192, 8, 4
    ctx = make_ctx(world_size=R, rank=rank, channels_per_rank=C, tile_order=order, xcd_swizzle=swz, group_m=gm)
    info = tl.tl_resolve(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    got = tl.tl_dump_schedule(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    want = omap.ag_gemm_schedule_records(M, N, K, R, C, rank, info["tile_m"], info["tile_n"], info["compute_workgroups"],
                                         rotate=(order == tl.TL_ORDER_RING), swizzle=bool(swz), group_m=info["group_m"])
    assert got == [v for rec in want for v in rec]
    assert info["expected_per_channel"] == omap.channel_expected(M, K, R, C, info["comm_tile_m"], info["comm_tile_n"])
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("rank,gm", [(5, 0), (0, 1), (7, 2)])
def test_arrival_order_schedule_matches_mapping_oracle(rank, gm):
    M, N, K, R, C = 8192, 3584, 8192, 8, 4
    ctx = make_ctx(world_size=R, rank=rank, channels_per_rank=C, tile_order=tl.TL_ORDER_ARRIVAL, xcd_swizzle=1, group_m=gm)
    info = tl.tl_resolve(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    got = tl.tl_dump_schedule(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    want = omap.ag_gemm_schedule_records(M, N, K, R, C, rank, info["tile_m"], info["tile_n"], info["compute_workgroups"],
                                         rotate=True, swizzle=True, group_m=info["group_m"], arrival=True)
    assert got == [v for rec in want for v in rec]
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("mode,order,kc", [("side", tl.TL_ORDER_ARRIVAL, 1), ("waves", tl.TL_ORDER_ARRIVAL, 2), ("side", tl.TL_ORDER_RING, 1)])
def test_arrival_order_and_paced_links(mode, order, kc):
    """Arrival tile order with the interleaved producer queue, with and without simulated links: same results, same
    flags.  400 GB/s per link: a 1 MiB shard takes 2.6 us, the call stays short."""
    w = wl.ag_gemm_inputs(2048, 456, 1024, 4, config_id=17)
    for gbps in (0, 400):
        hs, g, c, flags, info = run_ag_gemm(w, 2, 2, MODES[mode], epochs=2, tile_m=256, tile_n=256, tile_order=order, ag_k_chunks=kc,
                                            link_gbps=gbps, comm_workgroups=8)
        check(w, hs, g, c, f"order {order} {mode} k chunks {kc} links {gbps} GB/s")
        assert flags.tolist() == [2 * info["expected_per_channel"]] * (4 * 2 * info["k_chunks"])


@pytest.mark.parametrize("mode,order", [("side", tl.TL_ORDER_OWN_FIRST), ("side", tl.TL_ORDER_ARRIVAL), ("waves", tl.TL_ORDER_ARRIVAL)])
def test_late_producer_new_data_every_call(mode, order):
    """The producer is late on purpose (10 GB/s per link: a 1 MiB shard takes 105 us, the GEMM tiles of the remote rows
    are resident and waiting long before their rows arrive) and every call brings new shard contents into the same
    buffers: a tile that read any byte of the gathered matrix before its channel's flag would see the previous call's
    data and miss the oracle's result for this call's."""
    w = wl.ag_gemm_inputs(2048, 456, 1024, 4, config_id=19)
    hs, g, c, flags, info = run_ag_gemm(w, 1, 2, MODES[mode], epochs=3, tile_m=256, tile_n=256, tile_order=order, link_gbps=10, comm_workgroups=8)
    check(w, hs, g, c, f"late producer, {mode}, order {order}")
    assert flags.tolist() == [3 * info["expected_per_channel"]] * (4 * 2 * info["k_chunks"])


def test_paced_links_take_the_time_of_the_link():
    """Producers alone, 8 ranks, shards of 4 MiB at 50 GB/s per link: the gather may not finish before 4 MiB / 50 GB/s
    = 84 us have passed (all links run side by side), and does not take several times that either (warm calls)."""
    R, M, N, K = 8, 2048, 256, 8192
    w = wl.ag_gemm_inputs(M, N, K, R, config_id=18)
    ctx = make_ctx(world_size=R, rank=3, channels_per_rank=2, comm_mode=tl.TL_COMM_SIDE_KERNEL, comm_alone=1, link_gbps=50, tile_m=256, tile_n=256)
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    shards = [up(s) for s in w["a_shards"]]
    gathered, b, c = poison((M, K)), up(w["b"]), poison((M, N))
    flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    comm = torch.cuda.Stream()
    torch.cuda.synchronize()
    times = []
    for epoch in (1, 2, 3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(comm)
        tl.tl_ag_gemm(ctx, shards, gathered, b, c, M, N, K, flags, epoch, wsp, ws_bytes, torch.cuda.current_stream(), comm)
        e1.record(comm)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
        times.append(e0.elapsed_time(e1) * 1e3)
    tl.tl_ctx_destroy(ctx)
    assert np.array_equal(down(gathered), np.concatenate(w["a_shards"]))
    link_us = (M // R) * K * 2 / 50e9 * 1e6
    assert all(t >= link_us * 0.98 for t in times), (times, link_us)
    assert all(t <= link_us * 3 for t in times[1:]), (times, link_us)      # the first call also loads the kernel


def test_invalid_arguments_are_rejected_before_launch():
    ctx = make_ctx(world_size=4, rank=1, channels_per_rank=3)
    for dims in ([1023, 512, 512], [1024, 512, 100], [1024, 513, 512], [1024, 512, 512]):   # R∤M, K%8, N%8, C∤M/R
        with pytest.raises(tl.TileLinkError) as e:
            tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, dims)
        assert e.value.status == tl.TL_ERR_UNSUPPORTED_SHAPE
    with pytest.raises(tl.TileLinkError):
        tl.tl_ctx_create(world_size=2, rank=2, channels_per_rank=1)
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("mode,kc,rank", [("side", 2, 1), ("side", 4, 3), ("waves", 4, 0)])
def test_k_chunked_channels(mode, kc, rank):
    """AllGather channels cut into chunks along K, one flag per (channel, chunk): ragged N, several epochs with new data."""
    w = wl.ag_gemm_inputs(2048, 456, 2048, 4, config_id=15)
    hs, g, c, flags, info = run_ag_gemm(w, rank, 2, MODES[mode], epochs=3, tile_m=256, tile_n=256, ag_k_chunks=kc, comm_workgroups=8)
    assert info["k_chunks"] == kc and info["comm_tile_n"] == 2048 // kc
    check(w, hs, g, c, f"k chunks {kc} {mode}")
    assert flags.tolist() == [3 * info["expected_per_channel"]] * (4 * 2 * kc)


def test_k_chunks_fall_back_and_reject():
    # another tile shape or binding: one flag per channel, same results
    w = wl.ag_gemm_inputs(1024, 256, 1024, 4, config_id=16)
    hs, g, c, flags, info = run_ag_gemm(w, 0, 1, tl.TL_COMM_SIDE_KERNEL, tile_m=128, tile_n=128, ag_k_chunks=2)
    assert info["k_chunks"] == 1 and len(flags) == 4
    check(w, hs, g, c, "k chunks with the 128x128 tile")
    ctx = make_ctx(world_size=4, rank=0, comm_mode=tl.TL_COMM_SIDE_KERNEL, ag_k_chunks=4)
    with pytest.raises(tl.TileLinkError) as e:
        tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [1024, 256, 1024])     # 4 steps of 64 per chunk
    assert e.value.status == tl.TL_ERR_UNSUPPORTED_SHAPE
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("mode", ["waves", "side", "stream", "copy_engine"])
def test_full_size_tp8_share(mode):
    """BASELINE configuration 2: 8 shards of [1024,8192], B [8192,3584]; whole output compared, every binding with the
    grid the library picks by itself.  In `stream` mode the copies are kernels of the runtime that must become resident
    beside the persistent GEMM grid, so the library leaves compute units free for them; in `copy_engine` mode a DMA
    engine moves the shards and the GEMM grid keeps every compute unit."""
    w = wl.ag_gemm_inputs(8192, 3584, 8192, 8, config_id=2)
    a_ref, _, c_ref = ops.ag_gemm(w["a_shards"], w["b"])
    hs, g, c, flags, info = run_ag_gemm(w, 0, 4, MODES[mode], epochs=2)
    a_ref, _, c_ref = ops.ag_gemm(hs, w["b"])
    assert np.array_equal(g, a_ref)
    rel, mx = assert_close_bf16(c, c_ref, f"cfg2 {mode}")
    if mode == "copy_engine":
        assert info["compute_workgroups"] == torch.cuda.get_device_properties(0).multi_processor_count
    if mode in ("stream", "copy_engine"):
        assert flags.tolist() == [2] * 32
    print(f"cfg2 {mode}: tile {info['tile_m']}x{info['tile_n']} grid {info['compute_workgroups']} rel_fro={rel:.2e} max={mx:.2e}")


@pytest.mark.parametrize("kc,rank", [(1, 0), (4, 5)])
def test_full_size_tp8_share_bench_configuration(kc, rank):
    """The launch configuration bench.py times -- side-kernel producers, local shard in place, own-first tile order, four
    channels per rank, one flag per channel, rank 0 -- and the same with four chunks along K (bench.py --ag-k-chunks 4)."""
    w = wl.ag_gemm_inputs(8192, 3584, 8192, 8, config_id=2)
    hs, g, c, flags, info = run_ag_gemm(w, rank, 4, tl.TL_COMM_SIDE_KERNEL, epochs=2, in_place=True, tile_order=tl.TL_ORDER_OWN_FIRST, ag_k_chunks=kc)
    assert info["k_chunks"] == kc and (info["tile_m"], info["tile_n"]) == (256, 256)
    a_ref, _, c_ref = ops.ag_gemm(hs, w["b"])
    assert np.array_equal(g, a_ref)
    assert_close_bf16(c, c_ref, f"cfg2 side, in place, own first, {kc} K chunk(s), rank {rank}")
    assert flags.tolist() == [2 * info["expected_per_channel"]] * (8 * 4 * kc)


@pytest.mark.parametrize("rank,C,in_place", [(1, 2, False), (0, 1, True)])
def test_copy_engine_small(rank, C, in_place):
    """rank_copy_data on a copy engine + rank_notify behind every shard: three calls with fresh data."""
    w = wl.ag_gemm_inputs(1120, 456, 320, 4, config_id=19)
    hs, g, c, flags, info = run_ag_gemm(w, rank, C, tl.TL_COMM_COPY_ENGINE, epochs=3, in_place=in_place)
    check(w, hs, g, c, f"copy engine rank {rank} C {C}")
    assert flags.tolist() == [3] * (4 * C)
