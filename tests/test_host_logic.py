"""Host-side logic of the library without a GPU: a context made by tl_ctx_create_host answers the geometry queries and
the schedule dump (paper: "Tile-Centric Mapping"), which are compared with the mapping oracle here as the GPU tests do
on the device context; shapes the mapping cannot serve are refused before anything could be enqueued."""
import pytest

import paper_2503_20313_amd as tl
from oracle import mapping as omap

CUS = 256


def host_ctx(**kw):
    base = dict(world_size=1, rank=0, channels_per_rank=1, comm_mode=tl.TL_COMM_WAVES, tile_order=tl.TL_ORDER_RING, xcd_swizzle=1)
    base.update(kw)
    return tl.tl_ctx_create_host(CUS, **base)


def test_more_than_64_channels_are_refused():
    """The consumer's wait set is a 64-bit mask over the global channel index: R*C = 128 must not get through."""
    ctx = host_ctx(world_size=8, channels_per_rank=16)
    with pytest.raises(tl.TileLinkError) as e:
        tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [8192, 512, 512])
    assert e.value.status == tl.TL_ERR_UNSUPPORTED_SHAPE and "64" in str(e.value)
    tl.tl_ctx_destroy(ctx)
    ctx = host_ctx(world_size=8, channels_per_rank=8)      # exactly 64: fine
    assert tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [8192, 512, 512]) == (256, 64)
    tl.tl_ctx_destroy(ctx)


def test_k_rules():
    ctx = host_ctx(world_size=4)
    for K in (1376, 3696, 8, 4104):                        # multiples of 8: accepted, a short last K step is zero-filled
        tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [1024, 512, K])
        tl.tl_query_workspace(ctx, tl.TL_OP_GEMM_RS, [1024, 512, K])
    for K in (100, 3697, 4):
        with pytest.raises(tl.TileLinkError) as e:
            tl.tl_query_workspace(ctx, tl.TL_OP_GEMM_RS, [1024, 512, K])
        assert e.value.status == tl.TL_ERR_UNSUPPORTED_SHAPE
    tl.tl_ctx_destroy(ctx)


def test_host_context_cannot_launch():
    ctx = host_ctx(world_size=2)
    with pytest.raises(tl.TileLinkError) as e:
        tl.tl_ag_gemm(ctx, [0, 0], 0, 0, 0, 256, 512, 512, 0, 1, 0, 256)
    assert e.value.status == tl.TL_ERR_INVALID_ARG and "tl_ctx_create_host" in str(e.value)
    with pytest.raises(tl.TileLinkError):
        tl.tl_check_status(ctx, 0)
    tl.tl_ctx_destroy(ctx)
    with pytest.raises(tl.TileLinkError):
        tl.tl_ctx_create_host(0, world_size=2, rank=0, channels_per_rank=1)
    with pytest.raises(tl.TileLinkError):
        tl.tl_ctx_create_host(256, world_size=2, rank=2, channels_per_rank=1)


@pytest.mark.parametrize("rank,order,swz,gm", [(0, tl.TL_ORDER_RING, 1, 0), (5, tl.TL_ORDER_RING, 1, 8), (3, tl.TL_ORDER_NATURAL, 0, 1), (2, tl.TL_ORDER_RING, 0, 3)])
def test_ag_gemm_schedule_dump_matches_mapping_oracle(rank, order, swz, gm):
    M, N, K, R, C = 8192, 3584, 8192, 8, 4
    ctx = host_ctx(world_size=R, rank=rank, channels_per_rank=C, tile_order=order, xcd_swizzle=swz, group_m=gm)
    info = tl.tl_resolve(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    assert info["compute_workgroups"] == CUS
    got = tl.tl_dump_schedule(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    want = omap.ag_gemm_schedule_records(M, N, K, R, C, rank, info["tile_m"], info["tile_n"], info["compute_workgroups"],
                                         rotate=(order == tl.TL_ORDER_RING), swizzle=bool(swz), group_m=info["group_m"])
    assert got == [v for rec in want for v in rec]
    assert info["expected_per_channel"] == omap.channel_expected(M, K, R, C, info["comm_tile_m"], info["comm_tile_n"])
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("rank,gm", [(5, 0), (0, 1)])
def test_arrival_order_schedule_matches_mapping_oracle(rank, gm):
    M, N, K, R, C = 8192, 3584, 8192, 8, 4
    ctx = host_ctx(world_size=R, rank=rank, channels_per_rank=C, tile_order=tl.TL_ORDER_ARRIVAL, group_m=gm)
    info = tl.tl_resolve(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    got = tl.tl_dump_schedule(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    want = omap.ag_gemm_schedule_records(M, N, K, R, C, rank, info["tile_m"], info["tile_n"], info["compute_workgroups"],
                                         rotate=True, swizzle=True, group_m=info["group_m"], arrival=True)
    assert got == [v for rec in want for v in rec]
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("rank,order,swz", [(0, tl.TL_ORDER_RING, 1), (3, tl.TL_ORDER_NATURAL, 0), (5, tl.TL_ORDER_OWN_FIRST, 1)])
def test_gemm_rs_schedule_dump_matches_mapping_oracle(rank, order, swz):
    M, N, K, R = 8192, 8192, 3584, 8
    ctx = host_ctx(world_size=R, rank=rank, tile_order=order, xcd_swizzle=swz, comm_tile_m=128, comm_tile_n=512)
    info = tl.tl_resolve(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
    got = tl.tl_dump_schedule(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
    rot, own = order != tl.TL_ORDER_NATURAL, order == tl.TL_ORDER_OWN_FIRST
    gemm = omap.gemm_rs_schedule_records(M, N, K, R, rank, info["tile_m"], info["tile_n"], 128, 512, info["compute_workgroups"], rot, bool(swz),
                                         info["group_m"], own)
    table = omap.rs_tile_table(M, N, R, rank, info["tile_m"], info["tile_n"], 128, 512)
    want = [v for rec in gemm for v in rec]
    for t in omap.rs_consumer_order(M, N, R, rank, 128, 512, rot, own):
        cm, cn, rlo, rhi, clo, chi, dest, exp = table[t]
        want += [t, cm, cn, rlo, rhi, clo, chi, dest, exp]
    assert got == want
    tl.tl_ctx_destroy(ctx)


def test_moe_and_attention_geometry_queries():
    ctx = host_ctx(world_size=8, channels_per_rank=4, comm_mode=tl.TL_COMM_SIDE_KERNEL)
    q = tl.tl_moe_query(ctx, tl.TL_OP_MOE_AG_GATHER_GEMM, 8192, 4096, 1792, 32, 2)
    assert q["n_flags"] == 32 and q["tile_n"] in (128, 256) and q["max_row_tiles"] >= 16384 // q["tile_m"]
    tl.tl_ctx_destroy(ctx)
    ctx = host_ctx(world_size=8, rank=7, comm_mode=tl.TL_COMM_SIDE_KERNEL)
    a = tl.tl_attn_query(ctx, 32768, 32, 128, True)
    assert a["n_flags"] == 16 and a["shards_gathered"] == 8 and a["attention_workgroups"] == 16 * 32
    tl.tl_ctx_destroy(ctx)


def test_schedules_match_the_mapping_oracle_on_seeded_random_shapes():
    """200 seeded draws of (shape, world, channels, rank, tile, order, swizzle, group, grid size, compute units): every
    AllGather + GEMM and GEMM + ReduceScatter schedule the library dumps is the mapping oracle's, record by record -- whole
    and partial rounds, grids that are no multiple of the eight dies, ragged last tiles, every tile order."""
    import numpy as np
    rng = np.random.Generator(np.random.Philox(20313))
    tiles = [(256, 256), (256, 224), (128, 128)]
    checked = 0
    for _ in range(200):
        R = int(rng.choice([1, 2, 4, 8]))
        C = int(rng.choice([1, 2, 4]))
        tm, tn = tiles[int(rng.integers(len(tiles)))]
        rows_per_channel = int(rng.choice([64, 128, 256, 512]))
        M = R * C * rows_per_channel
        N = int(rng.integers(1, 40)) * 64 + int(rng.choice([0, 8, 200]))
        K = int(rng.integers(1, 64)) * 64
        rank = int(rng.integers(R))
        order = int(rng.choice([tl.TL_ORDER_NATURAL, tl.TL_ORDER_RING, tl.TL_ORDER_OWN_FIRST, tl.TL_ORDER_ARRIVAL]))
        swz, gm = int(rng.integers(2)), int(rng.choice([0, 1, 2, 3, 8]))
        cus = int(rng.choice([256, 64, 40, 304]))
        G = int(rng.choice([0, 0, 24, 100]))
        ctx = tl.tl_ctx_create_host(cus, world_size=R, rank=rank, channels_per_rank=C, comm_mode=tl.TL_COMM_SIDE_KERNEL, tile_order=order,
                                    xcd_swizzle=swz, group_m=gm, tile_m=tm, tile_n=tn, compute_workgroups=G)
        try:
            info = tl.tl_resolve(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
        except tl.TileLinkError:
            tl.tl_ctx_destroy(ctx)
            continue
        got = tl.tl_dump_schedule(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
        want = omap.ag_gemm_schedule_records(M, N, K, R, C, rank, info["tile_m"], info["tile_n"], info["compute_workgroups"],
                                             rotate=order != tl.TL_ORDER_NATURAL, swizzle=bool(swz), group_m=info["group_m"],
                                             arrival=order == tl.TL_ORDER_ARRIVAL)
        assert got == [v for rec in want for v in rec], (M, N, K, R, C, rank, tm, tn, order, swz, gm, cus, G)
        checked += 1
        if order != tl.TL_ORDER_ARRIVAL:
            try:
                info = tl.tl_resolve(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
            except tl.TileLinkError:
                tl.tl_ctx_destroy(ctx)
                continue
            got = tl.tl_dump_schedule(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
            rot, own = order != tl.TL_ORDER_NATURAL, order == tl.TL_ORDER_OWN_FIRST
            Tm_r, Tn_r = info["comm_tile_m"], info["comm_tile_n"]
            gemm = omap.gemm_rs_schedule_records(M, N, K, R, rank, info["tile_m"], info["tile_n"], Tm_r, Tn_r, info["compute_workgroups"], rot,
                                                 bool(swz), info["group_m"], own)
            table = omap.rs_tile_table(M, N, R, rank, info["tile_m"], info["tile_n"], Tm_r, Tn_r)
            want = [v for rec in gemm for v in rec]
            for t in omap.rs_consumer_order(M, N, R, rank, Tm_r, Tn_r, rot, own):
                cm, cn, rlo, rhi, clo, chi, dest, exp = table[t]
                want += [t, cm, cn, rlo, rhi, clo, chi, dest, exp]
            assert got == want, ("rs", M, N, K, R, C, rank, tm, tn, order, swz, gm, cus, G)
            checked += 1
        tl.tl_ctx_destroy(ctx)
    assert checked >= 150
