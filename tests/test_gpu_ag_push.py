"""GPU parity of tl_ag_gemm_push (AllGather + GEMM in push mode: the local shard is also delivered to every peer)
against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up

pytestmark = pytest.mark.gpu
MODES = {"waves": tl.TL_COMM_WAVES, "side": tl.TL_COMM_SIDE_KERNEL}


def run_push(w, rank, C, mode, epochs=1, in_place=False, **cfg):
    M, N, K, R = w["M"], w["N"], w["K"], w["world"]
    ctx = make_ctx(world_size=R, rank=rank, channels_per_rank=C, comm_mode=mode, **cfg)
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    info = tl.tl_resolve(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
    assert n_flags == R * C
    ms = M // R
    gathered = poison((M, K))
    shards = [up(s) for s in w["a_shards"]]
    if in_place:
        gathered[rank * ms:(rank + 1) * ms] = shards[rank]
        shards[rank] = gathered[rank * ms:(rank + 1) * ms]
    slots = [None if q == rank else poison((ms, K)) for q in range(R)]
    b, c = up(w["b"]), poison((M, N))
    flags = torch.zeros(2 * n_flags, dtype=torch.int32, device=dev())        # channel flags, then pushed counters
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    comm = torch.cuda.Stream()
    torch.cuda.synchronize()   # the fills above ran on the default stream; the communication stream does not order after it
    host_shards = [s.copy() for s in w["a_shards"]]
    for epoch in range(1, epochs + 1):
        if epoch > 1:
            for q in range(R):
                host_shards[q] = wl.normal_bf16(host_shards[q].shape, 1.0, 76, epoch, q)
                shards[q].copy_(up(host_shards[q]))
            c.copy_(poison((M, N)))
        torch.cuda.synchronize()
        tl.tl_ag_gemm_push(ctx, shards, gathered, [0 if t is None else t for t in slots], b, c, M, N, K, flags, epoch, wsp, ws_bytes,
                           torch.cuda.current_stream(), comm)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
    tl.tl_ctx_destroy(ctx)
    return host_shards, down(gathered), down(c), [None if t is None else down(t) for t in slots], flags.cpu().numpy(), info


def check(w, rank, C, epochs, hs, g, c, slots, flags, info, what):
    R = w["world"]
    a_ref, _, c_ref, slots_ref = ops.ag_gemm_push(hs, w["b"], rank)
    assert np.array_equal(g, a_ref), f"{what}: gathered A is not the concatenation of the shards"
    assert_close_bf16(c, c_ref, what)
    for q in range(R):
        if q != rank:
            assert np.array_equal(slots[q], slots_ref[q]), f"{what}: what peer {q} received is not this rank's shard"
    exp = epochs * info["expected_per_channel"]
    assert flags[:R * C].tolist() == [exp] * (R * C)
    pushed = flags[R * C:].reshape(R, C)
    for q in range(R):
        assert pushed[q].tolist() == ([0] if q == rank else [exp]) * C, f"{what}: pushed counters of peer {q}"


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("rank,C", [(0, 1), (1, 2), (3, 2)])
def test_small(mode, rank, C):
    w = wl.ag_gemm_inputs(512, 256, 256, 4, config_id=95)
    out = run_push(w, rank, C, MODES[mode], epochs=3, comm_workgroups=3)
    check(w, rank, C, 3, *out, f"push small {mode} rank={rank} C={C}")


def test_ragged_tiles_and_column_tiles():
    # 5 shards of 224 rows, producer tiles of 8 rows x 64 columns (5 column tiles), ragged GEMM tiles
    w = wl.ag_gemm_inputs(1120, 456, 320, 5, config_id=96)
    out = run_push(w, 2, 4, tl.TL_COMM_WAVES, epochs=2, tile_m=128, tile_n=128, comm_workgroups=3, comm_tile_m=8, comm_tile_n=64)
    check(w, 2, 4, 2, *out, "push ragged")


def test_producer_alone_and_rejections():
    w = wl.ag_gemm_inputs(512, 256, 256, 4, config_id=97)
    hs, g, c, slots, flags, info = run_push(w, 1, 2, tl.TL_COMM_SIDE_KERNEL, comm_alone=1, comm_workgroups=2)
    assert np.array_equal(g, ops.all_gather_rows(hs)) and all(np.array_equal(slots[q], hs[1]) for q in (0, 2, 3))
    assert (c == 0x7FC0).all()                                  # no GEMM in this mode
    ctx = make_ctx(world_size=2, rank=0, comm_mode=tl.TL_COMM_STREAM)
    w = wl.ag_gemm_inputs(256, 256, 128, 2, config_id=97)
    shards = [up(s) for s in w["a_shards"]]
    flags = torch.zeros(64, dtype=torch.int32, device=dev())
    wsp = torch.zeros(64, dtype=torch.int32, device=dev())
    args = (shards, poison((256, 128)), [0, poison((128, 128))], up(w["b"]), poison((256, 256)), 256, 256, 128, flags, 1, wsp, 256)
    with pytest.raises(tl.TileLinkError) as e:                  # the copy-engine binding has no push form
        tl.tl_ag_gemm_push(ctx, *args)
    assert e.value.status == tl.TL_ERR_INVALID_ARG
    tl.tl_ctx_destroy(ctx)
    ctx = make_ctx(world_size=2, rank=0, comm_mode=tl.TL_COMM_WAVES)
    with pytest.raises(tl.TileLinkError) as e:                  # the peer's slot is missing
        tl.tl_ag_gemm_push(ctx, shards, args[1], [0, 0], *args[3:])
    assert e.value.status == tl.TL_ERR_INVALID_ARG
    torch.cuda.synchronize()
    tl.tl_ctx_destroy(ctx)


def test_full_size_mlp5_share():
    """MLP-5 part 1 at TP=8 in push mode: sampled output columns; every peer's slot is the local shard bit for bit."""
    M, N, K, R, rank = 8192, 3584, 8192, 8, 3
    w = wl.ag_gemm_inputs(M, N, K, R, config_id=98)
    hs, g, c, slots, flags, info = run_push(w, rank, 4, tl.TL_COMM_SIDE_KERNEL, in_place=True, tile_order=tl.TL_ORDER_OWN_FIRST)
    rng = np.random.Generator(np.random.Philox(980))
    cols = np.array(sorted(set(range(8)) | set(range(N - 8, N)) | set(rng.choice(N, size=256, replace=False).tolist())))
    a_ref, _, c_ref = ops.ag_gemm(hs, np.ascontiguousarray(w["b"][:, cols]))
    assert np.array_equal(g, a_ref)
    assert_close_bf16(c[:, cols], c_ref, "push MLP-5 share")
    for q in range(R):
        if q != rank:
            assert np.array_equal(slots[q], hs[rank])
    exp = info["expected_per_channel"]
    assert flags[:R * 4].tolist() == [exp] * (R * 4)
    assert flags[R * 4:].reshape(R, 4).sum(axis=1).tolist() == [0 if q == rank else 4 * exp for q in range(R)]
