"""GPU parity of tl_gemm_ring_rs (GEMM + ring ReduceScatter, one rank of the ring) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from oracle.bf16 import round_to_bf16, widen
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up

pytestmark = pytest.mark.gpu

MODES = {"waves": tl.TL_COMM_WAVES, "side": tl.TL_COMM_SIDE_KERNEL, "stream": tl.TL_COMM_STREAM}


def run_ring(w, mode, epochs=1, **cfg):
    M, N, K, R, rank = w["M"], w["N"], w["K"], w["world"], w["rank"]
    ctx = make_ctx(world_size=R, rank=rank, comm_mode=mode, **cfg)
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
    info = tl.tl_resolve(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
    seg = M // R
    a, b = up(w["a"]), up(w["b"])
    partial = poison((M, N))
    recv = [0 if t is None else up(t) for t in w["ring_recv"]]
    push = [None if q == rank else poison((seg, N)) for q in range(R)]
    out = poison((seg, N))
    flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    comm = torch.cuda.Stream()
    torch.cuda.synchronize()   # the fills above ran on the default stream; the communication stream does not order after it
    host_a = w["a"]
    for epoch in range(1, epochs + 1):
        if epoch > 1:
            host_a = wl.normal_bf16(host_a.shape, 1.0, 77, epoch)
            a.copy_(up(host_a))
            out.copy_(poison((seg, N)))
        torch.cuda.synchronize()
        tl.tl_gemm_ring_rs(ctx, a, b, partial, recv, [0 if t is None else t for t in push], out, M, N, K, flags, epoch, wsp, ws_bytes,
                           torch.cuda.current_stream(), comm)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
    tl.tl_ctx_destroy(ctx)
    return host_a, down(partial), [None if t is None else down(t) for t in push], down(out), flags.cpu().numpy(), info


def one_ulp(got, exact, what):
    diff = np.abs(widen(got) - widen(exact))
    assert np.all(diff <= np.abs(widen(exact)) * 2.0 ** -7 + 1e-30), f"{what}: differs by more than one bf16 ulp"
    assert np.mean(got != exact) < 0.02, f"{what}: too many last-bit differences"


def check(w, host_a, partial, push, out, what):
    R, rank = w["world"], w["rank"]
    seg = w["M"] // R
    p_ref, passed_ref, out_ref = ops.gemm_ring_rs(host_a, w["b"], w["ring_recv"], rank)
    assert_close_bf16(partial, p_ref, what + " partial")
    start = (rank + 1) % R
    # the hops of the GPU's own partial, recomputed by the oracle: a tight check of the reduce side (the sum of two bf16
    # values rounded through fp32 may differ from the exactly rounded one in the last bit, rarely)
    passed_own, out_own = ops.ring_rs_rank(partial, w["ring_recv"], rank)
    for q in range(R):
        if q == rank:
            continue
        if q == start:
            assert np.array_equal(push[q], partial[q * seg:(q + 1) * seg]), f"{what}: the chain of segment {q} must start with the partial rows"
        else:
            one_ulp(push[q], passed_own[q], f"{what}: running sum of segment {q}")
        assert_close_bf16(push[q], passed_ref[q], f"{what}: running sum of segment {q}")
    if R > 1:
        one_ulp(out, out_own, what + ": own segment")
    else:
        assert np.array_equal(out, partial)
    return assert_close_bf16(out, out_ref, what + " out")


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("rank", [0, 1, 3])
def test_small(mode, rank):
    w = wl.gemm_ring_rs_inputs(512, 512, 256, 4, rank, config_id=81)
    ha, partial, push, out, flags, info = run_ring(w, MODES[mode], epochs=3, comm_workgroups=3)
    check(w, ha, partial, push, out, f"ring small {mode} r={rank}")
    n_rt = info["n_comm_tiles"]
    tps = n_rt // 4
    ready, arrived, pushed = flags[:n_rt], flags[n_rt:n_rt + 4 * tps], flags[n_rt + 4 * tps:]
    start = (rank + 1) % 4
    assert ready.tolist() == [3] * n_rt
    for q in range(4):
        assert arrived[q * tps:(q + 1) * tps].tolist() == ([0] if q == start else [3]) * tps    # nothing arrives for the chain that starts here
        assert pushed[q * tps:(q + 1) * tps].tolist() == ([0] if q == rank else [3]) * tps      # the own segment is not passed on


def test_ragged_tiles_and_natural_order():
    # 5 ranks of 224 rows, N = 320: GEMM tiles straddle segments, ragged last column tile; explicit small reduce tiles
    w = wl.gemm_ring_rs_inputs(1120, 320, 192, 5, 2, config_id=82)
    ha, partial, push, out, _, _ = run_ring(w, tl.TL_COMM_WAVES, epochs=2, comm_workgroups=3, tile_m=128, tile_n=128, comm_tile_m=32, comm_tile_n=64)
    check(w, ha, partial, push, out, "ring ragged waves")
    ha, partial, push, out, _, _ = run_ring(w, tl.TL_COMM_SIDE_KERNEL, comm_workgroups=4, tile_order=tl.TL_ORDER_NATURAL, comm_tile_m=56)
    check(w, ha, partial, push, out, "ring ragged side, natural order")


def test_single_rank_and_direct_push_ignored():
    w = wl.gemm_ring_rs_inputs(256, 256, 128, 1, 0, config_id=83)
    ha, partial, push, out, _, _ = run_ring(w, tl.TL_COMM_WAVES, comm_workgroups=2)
    check(w, ha, partial, push, out, "ring of one rank")
    w = wl.gemm_ring_rs_inputs(256, 256, 128, 2, 1, config_id=83)
    ha, partial, push, out, _, _ = run_ring(w, tl.TL_COMM_SIDE_KERNEL, comm_workgroups=2, rs_direct_push=2)
    check(w, ha, partial, push, out, "ring, direct push requested")


def test_reduce_side_alone_on_a_finished_partial():
    """comm_alone: the ring's reduce side runs on a partial product that a call without communication left behind."""
    w = wl.gemm_ring_rs_inputs(512, 256, 128, 4, 2, config_id=86)
    M, N, K, R, rank = 512, 256, 128, 4, 2
    seg = M // R
    a, b = up(w["a"]), up(w["b"])
    partial, out = poison((M, N)), poison((seg, N))
    recv = [0 if t is None else up(t) for t in w["ring_recv"]]
    push = [None if q == rank else poison((seg, N)) for q in range(R)]
    push_arg = [0 if t is None else t for t in push]
    comm = torch.cuda.Stream()
    for mode, alone in ((tl.TL_COMM_NONE, 0), (tl.TL_COMM_SIDE_KERNEL, 1)):
        ctx = make_ctx(world_size=R, rank=rank, comm_mode=mode, comm_alone=alone, comm_workgroups=3)
        ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_GEMM_RS, [M, N, K])
        flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
        wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
        torch.cuda.synchronize()
        tl.tl_gemm_ring_rs(ctx, a, b, partial, recv, push_arg, out, M, N, K, flags, 1, wsp, ws_bytes, torch.cuda.current_stream(), comm)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
        tl.tl_ctx_destroy(ctx)
        if not alone:
            assert (down(out) == 0x7FC0).all()          # no reduce side in this mode
    check(w, w["a"], down(partial), [None if t is None else down(t) for t in push], down(out), "ring reduce side alone")


def test_rejects_missing_buffers():
    ctx = make_ctx(world_size=2, rank=0, comm_mode=tl.TL_COMM_WAVES)
    w = wl.gemm_ring_rs_inputs(256, 256, 128, 2, 0, config_id=84)
    ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_GEMM_RS, [256, 256, 128])
    flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
    wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
    a, b, partial, out, buf = up(w["a"]), up(w["b"]), poison((256, 256)), poison((128, 256)), poison((128, 256))
    with pytest.raises(tl.TileLinkError) as e:      # the own segment's incoming running sum is needed (entry 0), entry 1 is not
        tl.tl_gemm_ring_rs(ctx, a, b, partial, [0, buf], [0, buf], out, 256, 256, 128, flags, 1, wsp, ws_bytes)
    assert e.value.status == tl.TL_ERR_INVALID_ARG
    with pytest.raises(tl.TileLinkError) as e:      # the landing zone of segment 1 is needed
        tl.tl_gemm_ring_rs(ctx, a, b, partial, [buf, 0], [0, 0], out, 256, 256, 128, flags, 1, wsp, ws_bytes)
    assert e.value.status == tl.TL_ERR_INVALID_ARG
    torch.cuda.synchronize()
    tl.tl_ctx_destroy(ctx)


def test_full_size_mlp5_share():
    """MLP-5 part 2 at TP=8 as a ring: sampled rows of every segment (the oracle computes those rows of the product only)."""
    M, N, K, R, rank = 8192, 8192, 3584, 8, 5
    w = wl.gemm_ring_rs_inputs(M, N, K, R, rank, config_id=85)
    ha, partial, push, out, flags, info = run_ring(w, tl.TL_COMM_SIDE_KERNEL, tile_order=tl.TL_ORDER_RING)
    seg = M // R
    rng = np.random.Generator(np.random.Philox(850))
    local = np.array(sorted({0, 1, seg - 1} | set(rng.choice(seg, size=13, replace=False).tolist())))
    rows = np.concatenate([q * seg + local for q in range(R)])
    p_rows = round_to_bf16(widen(ha[rows]) @ widen(w["b"]))
    assert_close_bf16(partial[rows], p_rows, "ring MLP-5 partial (sampled rows)")
    start = (rank + 1) % R
    for q in range(R):
        own = p_rows[q * len(local):(q + 1) * len(local)]
        want = ops.ring_hop(own, None if q == start else w["ring_recv"][q][local])
        got = out[local] if q == rank else push[q][local]
        assert_close_bf16(got, want, f"ring MLP-5 segment {q}")
    assert not (out == 0x7FC0).any() and all(not (push[q] == 0x7FC0).any() for q in range(R) if q != rank)
    n_rt = info["n_comm_tiles"]
    assert (flags[:n_rt] > 0).all()
