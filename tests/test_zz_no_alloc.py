"""tl_ag_gemm_static, the entry point for callers that cannot allocate: its results against those of tl_ag_gemm (same
kernels, caller-owned workspace) on two calls in a row, the second with a smaller input, through the C ABI.  Runs last:
every test shares the one static scratch array of the device."""
import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up
from tests.test_gpu_ag_gemm import run_ag_gemm

pytestmark = pytest.mark.gpu
MODES = {"waves": tl.TL_COMM_WAVES, "side": tl.TL_COMM_SIDE_KERNEL, "copy_engine": tl.TL_COMM_COPY_ENGINE}
# (M, N, K, R, C, rank): the second call is smaller in every dimension and has fewer flags
CALLS = [(2048, 456, 1040, 4, 2, 1), (256, 512, 512, 2, 1, 0)]


@pytest.mark.parametrize("mode", list(MODES))
def test_two_calls_in_a_row_match_the_workspace_entry_point(mode):
    cfg = dict(comm_mode=MODES[mode], comm_workgroups=4, tile_order=tl.TL_ORDER_OWN_FIRST)
    want = []
    for i, (M, N, K, R, C, rank) in enumerate(CALLS):
        w = wl.ag_gemm_inputs(M, N, K, R, config_id=130 + i)
        hs, g, c, flags, info = run_ag_gemm(w, rank, C, MODES[mode], **{k: v for k, v in cfg.items() if k != "comm_mode"})
        want.append((w, g, c))
    cs, ms = torch.cuda.Stream(), torch.cuda.Stream()
    got = []
    for i, (M, N, K, R, C, rank) in enumerate(CALLS):
        w = want[i][0]
        ctx = make_ctx(world_size=R, rank=rank, channels_per_rank=C, **cfg)
        shards = [up(s) for s in w["a_shards"]]
        gathered, b, c = poison((M, K)), up(w["b"]), poison((M, N))
        torch.cuda.synchronize()
        tl.tl_ag_gemm_static(ctx, shards, gathered, b, c, M, N, K, cs, ms)
        torch.cuda.synchronize()
        tl.tl_check_status(ctx, None)
        tl.tl_ctx_destroy(ctx)
        got.append((down(gathered), down(c)))
    for i, ((w, g_ref, c_ref), (g, c)) in enumerate(zip(want, got)):
        assert np.array_equal(g, g_ref), f"call {i}: gathered matrix"
        assert np.array_equal(c, c_ref), f"call {i}: product differs from tl_ag_gemm's (same kernels: bit for bit)"
        _, _, c_oracle = ops.ag_gemm(w["a_shards"], w["b"])
        assert_close_bf16(c, c_oracle, f"static call {i} {mode}")


def test_repeated_calls_on_the_same_buffers_and_default_streams():
    """Five calls back to back on the default stream without a synchronisation in between, fresh shard data before the
    last one: the scratch is cleared by every call, in stream order."""
    M, N, K, R, C, rank = 1024, 256, 512, 4, 2, 2
    w = wl.ag_gemm_inputs(M, N, K, R, config_id=132)
    ctx = make_ctx(world_size=R, rank=rank, channels_per_rank=C, comm_mode=tl.TL_COMM_WAVES, comm_workgroups=2)
    shards = [up(s) for s in w["a_shards"]]
    gathered, b, c = poison((M, K)), up(w["b"]), poison((M, N))
    for _ in range(4):
        tl.tl_ag_gemm_static(ctx, shards, gathered, b, c, M, N, K)
    fresh = [wl.normal_bf16(s.shape, 1.0, 133, 0, q) for q, s in enumerate(w["a_shards"])]
    for q in range(R):
        shards[q].copy_(up(fresh[q]))
    tl.tl_ag_gemm_static(ctx, shards, gathered, b, c, M, N, K)
    torch.cuda.synchronize()
    tl.tl_check_status(ctx, None)
    tl.tl_ctx_destroy(ctx)
    a_ref, _, c_ref = ops.ag_gemm(fresh, w["b"])
    assert np.array_equal(down(gathered), a_ref)
    assert_close_bf16(down(c), c_ref, "static, fifth call")


def test_sizes_beyond_the_static_scratch_are_refused():
    ctx = make_ctx(world_size=8, rank=0, channels_per_rank=8, comm_mode=tl.TL_COMM_SIDE_KERNEL, tile_m=256, tile_n=256, ag_k_chunks=128)
    with pytest.raises(tl.TileLinkError) as e:
        tl.tl_ag_gemm_static(ctx, [0] * 8, 0, 0, 0, 16384, 512, 65536)      # 8 x 8 x 128 = 8192 flags
    assert e.value.status == tl.TL_ERR_WORKSPACE_TOO_SMALL and "4096" in str(e.value)
    tl.tl_ctx_destroy(ctx)
