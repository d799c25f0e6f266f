"""GPU parity of tl_sp_ag_attention (AllGather of K/V overlapped with flash attention of the local queries)
against the CPU oracle, through the C ABI."""
import math

import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up

pytestmark = pytest.mark.gpu
MODES = {"none": tl.TL_COMM_NONE, "waves": tl.TL_COMM_WAVES, "side": tl.TL_COMM_SIDE_KERNEL, "copy_engine": tl.TL_COMM_COPY_ENGINE}
POISON = 0x7FC0


def run_attention(w, rank, causal, mode, C=1, epochs=1, scale=None, k_std=None, **cfg):
    S, Hd, D, R = w["S"], w["heads"], w["head_dim"], w["world"]
    S_loc = S // R
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    ctx = make_ctx(world_size=R, rank=rank, channels_per_rank=C, comm_mode=mode, **cfg)
    info = tl.tl_attn_query(ctx, S, Hd, D, causal)
    q = up(w["q_shards"][rank])
    ks = [up(s) for s in w["k_shards"]]
    vs = [up(s) for s in w["v_shards"]]
    if mode == tl.TL_COMM_NONE:   # the gathered buffers are inputs
        kg = up(ops.all_gather_rows(w["k_shards"]))
        vg = up(ops.all_gather_rows(w["v_shards"]))
    else:
        kg, vg = poison((S, Hd, D)), poison((S, Hd, D))
    o = poison((S_loc, Hd, D))
    flags = torch.zeros(info["n_flags"], dtype=torch.int32, device=dev())
    wsp = torch.zeros(info["ws_bytes"] // 4, dtype=torch.int32, device=dev())
    comm = torch.cuda.Stream()
    torch.cuda.synchronize()   # the zero fills above ran on the default stream; the communication stream does not order after it
    for epoch in range(1, epochs + 1):
        if epoch > 1:   # new keys and values every call: a stale flag would let old data through
            for r_ in range(R):
                w["k_shards"][r_] = wl.normal_bf16((S_loc, Hd, D), 1.0, 91, epoch, r_)
                w["v_shards"][r_] = wl.normal_bf16((S_loc, Hd, D), 1.0, 92, epoch, r_)
                ks[r_].copy_(up(w["k_shards"][r_]))
                vs[r_].copy_(up(w["v_shards"][r_]))
            o.copy_(poison((S_loc, Hd, D)))
            torch.cuda.synchronize()
        tl.tl_sp_ag_attention(ctx, q, ks, vs, kg, vg, o, S, Hd, D, causal, scale, flags, epoch, wsp, info["ws_bytes"],
                              torch.cuda.current_stream(), comm)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, wsp)
    res = dict(o=down(o), kg=down(kg), vg=down(vg), flags=flags.cpu().numpy().astype(np.int64), info=info, scale=scale)
    tl.tl_ctx_destroy(ctx)
    return res


def check_gathered(w, res, rank, causal, C, epochs=1):
    R = w["world"]
    S_loc = w["S"] // R
    need = rank + 1 if causal else R
    k_ref, v_ref = ops.all_gather_rows(w["k_shards"]), ops.all_gather_rows(w["v_shards"])
    assert np.array_equal(res["kg"][: need * S_loc], k_ref[: need * S_loc])
    assert np.array_equal(res["vg"][: need * S_loc], v_ref[: need * S_loc])
    if need < R and epochs == 1:   # shards a causal rank never reads are not copied
        assert (res["kg"][need * S_loc:] == POISON).all() and (res["vg"][need * S_loc:] == POISON).all()
    exp = np.zeros(2 * R * C, dtype=np.int64)
    e = res["info"]["expected_per_channel"] * epochs
    exp[: need * C] = e
    exp[R * C: R * C + need * C] = e
    assert np.array_equal(res["flags"], exp)


@pytest.mark.parametrize("mode", ["none", "waves", "side", "copy_engine"])
@pytest.mark.parametrize("causal", [True, False])
def test_small(mode, causal):
    w = wl.sp_attention_inputs(512, 2, 128, 2, config_id=51)
    for rank in range(2):
        res = run_attention(w, rank, causal, MODES[mode])
        _, _, _, o_ref = ops.sp_ag_attention(w["q_shards"][rank], w["k_shards"], w["v_shards"], rank, causal)
        assert_close_bf16(res["o"], o_ref, f"attention small rank {rank} {mode} causal={causal}")
        if mode != "none":
            check_gathered(w, res, rank, causal, 1)


@pytest.mark.parametrize("S,heads,R,C,rank,causal,mode", [
    (768, 3, 4, 1, 2, True, "waves"),      # S/R = 192: ragged query block (192 of 256), heads not a multiple of 8
    (1920, 1, 3, 2, 1, True, "side"),      # S/R = 640 = 2.5 query blocks, two channels per rank
    (1920, 2, 3, 5, 2, False, "waves"),    # channels of 128 rows
    (1024, 8, 8, 2, 7, True, "side"),      # last rank: every shard needed
    (1024, 8, 8, 1, 0, True, "waves"),     # first rank: only the local shard
    (2048, 16, 4, 4, 3, False, "side"),
])
def test_shapes(S, heads, R, C, rank, causal, mode):
    w = wl.sp_attention_inputs(S, heads, 128, R, config_id=52)
    res = run_attention(w, rank, causal, MODES[mode], C=C)
    _, _, _, o_ref = ops.sp_ag_attention(w["q_shards"][rank], w["k_shards"], w["v_shards"], rank, causal)
    assert_close_bf16(res["o"], o_ref, f"attention S={S} heads={heads} R={R} C={C} rank={rank}")
    check_gathered(w, res, rank, causal, C)


@pytest.mark.parametrize("rank,mode,C", [(3, "side", 2), (0, "waves", 1), (2, "waves", 2)])
def test_simulated_links(rank, mode, C):
    """K and V shards arriving over simulated links (interleaved producer queue, paced tiles, consumers that only wait):
    same result.  800 GB/s: a 128 KiB shard pair takes a fraction of a microsecond, the call stays short."""
    w = wl.sp_attention_inputs(1024, 4, 128, 4, config_id=56)
    res = run_attention(w, rank, True, MODES[mode], C=C, epochs=2, link_gbps=800)
    _, _, _, o_ref = ops.sp_ag_attention(w["q_shards"][rank], w["k_shards"], w["v_shards"], rank, True)
    assert_close_bf16(res["o"], o_ref, f"attention over simulated links rank {rank} {mode}")
    check_gathered(w, res, rank, True, C, epochs=2)


def test_peaked_scores_and_scale():
    """Large score spread (scale 4x the usual one): the running maximum moves a lot, old partial sums are rescaled
    by tiny factors, and most probabilities underflow to zero."""
    w = wl.sp_attention_inputs(1024, 2, 128, 2, config_id=53)
    scale = 4.0 / math.sqrt(128)
    res = run_attention(w, 1, True, tl.TL_COMM_WAVES, scale=scale)
    _, _, _, o_ref = ops.sp_ag_attention(w["q_shards"][1], w["k_shards"], w["v_shards"], 1, True, scale=scale)
    assert_close_bf16(res["o"], o_ref, "attention with peaked scores")


def test_single_key_rows():
    """Rank 0, causal: query 0 sees exactly one key, so its output row is that value row (softmax of one element)."""
    w = wl.sp_attention_inputs(512, 2, 128, 2, config_id=54)
    res = run_attention(w, 0, True, tl.TL_COMM_WAVES)
    assert np.array_equal(res["o"][0], w["v_shards"][0][0])


@pytest.mark.parametrize("mode", ["waves", "side", "copy_engine"])
def test_epochs_reuse_flags(mode):
    w = wl.sp_attention_inputs(1024, 4, 128, 4, config_id=55)
    res = run_attention(w, 2, True, MODES[mode], C=2, epochs=3)
    _, _, _, o_ref = ops.sp_ag_attention(w["q_shards"][2], w["k_shards"], w["v_shards"], 2, True)
    assert_close_bf16(res["o"], o_ref, "attention third call")
    check_gathered(w, res, 2, True, 2, epochs=3)


def test_drained_queue_times_out():
    """A wait that can never be satisfied must end with TL_ERR_TIMEOUT instead of hanging.  Forced from the host: the two
    producer queue heads start far past the end of this call's queue, so nobody copies or notifies anything."""
    w = wl.sp_attention_inputs(512, 1, 128, 2, config_id=56)
    S, Hd, D, R = 512, 1, 128, 2
    ctx = make_ctx(world_size=R, rank=1, comm_mode=tl.TL_COMM_WAVES, spin_timeout_us=20_000)
    info = tl.tl_attn_query(ctx, S, Hd, D, True)
    q = up(w["q_shards"][1])
    ks = [up(s) for s in w["k_shards"]]
    vs = [up(s) for s in w["v_shards"]]
    kg, vg, o = poison((S, Hd, D)), poison((S, Hd, D)), poison((S // R, Hd, D))
    flags = torch.zeros(info["n_flags"], dtype=torch.int32, device=dev())
    wsp = torch.zeros(info["ws_bytes"] // 4, dtype=torch.int32, device=dev())
    wsp[1] = 1 << 20
    wsp[2] = 1 << 20
    torch.cuda.synchronize()
    tl.tl_sp_ag_attention(ctx, q, ks, vs, kg, vg, o, S, Hd, D, True, 1.0 / math.sqrt(D), flags, 1, wsp, info["ws_bytes"],
                          torch.cuda.current_stream(), torch.cuda.Stream())
    torch.cuda.synchronize()
    with pytest.raises(tl.TileLinkError) as ei:
        tl.tl_check_status(ctx, wsp)
    assert ei.value.status == tl.TL_ERR_TIMEOUT
    assert int(flags.abs().sum().item()) == 0
    tl.tl_ctx_destroy(ctx)


def test_invalid_arguments():
    ctx = make_ctx(world_size=2, rank=0)
    with pytest.raises(tl.TileLinkError):
        tl.tl_attn_query(ctx, 512, 2, 64, True)       # head_dim
    with pytest.raises(tl.TileLinkError):
        tl.tl_attn_query(ctx, 513, 2, 128, True)      # R does not divide S
    with pytest.raises(tl.TileLinkError):
        tl.tl_attn_query(ctx, 2 * 96, 2, 128, True)   # rows per channel not a multiple of 64
    tl.tl_ctx_destroy(ctx)


@pytest.mark.parametrize("rank,mode", [(7, "side"), (3, "waves"), (0, "side"), (7, "copy_engine")])
def test_full_size_sampled(rank, mode):
    """Config 5 (S=32768, 32 heads, head_dim 128, TP=8, causal) in the launch configuration the bench uses.  The oracle
    computes EVERY head on rows of EVERY one of the 16 query blocks (a workgroup owns one head and 256 queries, a wave 32
    of them): each block's first and last rows, the rows either side of its wave boundaries at 32, 128 and 224, and one
    row inside -- 160 rows x 32 heads, so an indexing slip per head, per query block or per wave would meet the oracle."""
    c = wl.CONFIGS[5]
    w = wl.sp_attention_inputs(c["S"], c["heads"], c["head_dim"], c["world"])
    res = run_attention(w, rank, True, MODES[mode])
    S_loc = c["S"] // c["world"]
    in_block = [0, 1, 31, 32, 77, 127, 128, 223, 224, 255]
    rows = np.array([256 * b + i for b in range(S_loc // 256) for i in in_block])
    heads = list(range(c["heads"]))
    _, _, _, o_ref = ops.sp_ag_attention(w["q_shards"][rank], w["k_shards"], w["v_shards"], rank, True, heads=heads, rows=rows)
    got = res["o"][rows][:, heads]
    assert_close_bf16(got, o_ref, f"attention full size rank {rank} {mode}")
    for h in heads:                                   # no head may hide behind the others' norm
        assert_close_bf16(got[:, h], o_ref[:, h], f"attention full size rank {rank} {mode} head {h}")
    for b in range(S_loc // 256):                     # ... and no query block
        sl = slice(b * len(in_block), (b + 1) * len(in_block))
        assert_close_bf16(got[sl], o_ref[sl], f"attention full size rank {rank} {mode} query block {b}")
    check_gathered(w, res, rank, True, 1)
    assert not (res["o"] == POISON).any()
