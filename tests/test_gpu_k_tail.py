"""GPU parity for reduction lengths K that are not a multiple of the tile kernels' K step (32): the short last step is
filled up with zeros inside the kernel.  The shares of the paper's benchmark table with such K (MLP-1: I/8 = 1376 = 43
steps of 32; MLP-6: I/8 = 3696 = 115 steps and a half) are in test_gpu_other_shapes.py; here small cases span every
tile shape, every length of the tail, and operands whose neighbourhood in memory is NaN."""
import numpy as np
import pytest
import torch

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from oracle.bf16 import round_to_bf16
from tests.gpu_util import assert_close_bf16, dev, down, make_ctx, poison, up
from tests.test_gpu_ag_gemm import check as check_ag
from tests.test_gpu_ag_gemm import run_ag_gemm
from tests.test_gpu_gemm_rs import check as check_rs
from tests.test_gpu_gemm_rs import run_gemm_rs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("tile", [(256, 256), (256, 224), (128, 128)])
@pytest.mark.parametrize("K", [8, 24, 40, 104, 1040])
def test_ag_gemm_k_tail(tile, K):
    # 4 shards of 280 rows, N = 456: ragged in M and N as well; K = 8 and 24 are a single short step, 40 = one step + 8,
    # 104 = three steps + 8, 1040 = 32 steps + 16
    w = wl.ag_gemm_inputs(1120, 456, K, 4, config_id=110)
    hs, g, c, flags, info = run_ag_gemm(w, 1, 2, tl.TL_COMM_WAVES, epochs=2, tile_m=tile[0], tile_n=tile[1], comm_workgroups=3)
    assert (info["tile_m"], info["tile_n"]) == tile
    check_ag(w, hs, g, c, f"K tail K={K} tile={tile}")


@pytest.mark.parametrize("K,direct", [(8, 0), (72, 1), (1040, 2), (1376, 1)])
def test_gemm_rs_k_tail(K, direct):
    w = wl.gemm_rs_inputs(1120, 456, K, 4, 1, config_id=111)
    ha, partial, push, out, flags, info = run_gemm_rs(w, tl.TL_COMM_SIDE_KERNEL, epochs=2, comm_workgroups=3, rs_direct_push=direct)
    check_rs(w, ha, partial, push, out, f"GEMM+RS K tail K={K} direct={direct}", direct=bool(direct))


@pytest.mark.parametrize("K", [8, 48, 88, 120])
def test_exact_integers_with_nan_beyond_the_operands(K):
    """Integer-valued operands (every partial sum exact in fp32: bit-exact result) that sit in larger buffers filled with
    NaN: the 16-byte pieces of the short last K step that lie beyond K -- the start of A's next row, or beyond A's last
    row; rows of B beyond its last -- may not reach the product, and a NaN times a zero would show."""
    g = np.random.default_rng(K)
    M, N = 384, 264
    a = round_to_bf16(g.integers(-3, 4, size=(M, K)).astype(np.float64))
    b = round_to_bf16(g.integers(-2, 3, size=(K, N)).astype(np.float64))
    a_big, b_big = poison((M + 8, K)), poison((K + 40, N))
    a_big[:M].copy_(up(a))
    b_big[:K].copy_(up(b))
    for tile in ((256, 256), (128, 128)):
        ctx = make_ctx(world_size=2, rank=0, comm_mode=tl.TL_COMM_NONE, tile_m=tile[0], tile_n=tile[1])
        ws_bytes, n_flags = tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [M, N, K])
        c = poison((M, N))
        flags = torch.zeros(n_flags, dtype=torch.int32, device=dev())
        wsp = torch.zeros(ws_bytes // 4, dtype=torch.int32, device=dev())
        shards = [a_big[:M // 2], a_big[M // 2:M]]
        torch.cuda.synchronize()
        tl.tl_ag_gemm(ctx, shards, a_big, b_big, c, M, N, K, flags, 1, wsp, ws_bytes)
        torch.cuda.synchronize()
        tl.tl_ctx_destroy(ctx)
        _, _, c_ref = ops.ag_gemm([a[:M // 2], a[M // 2:]], b)
        assert np.array_equal(down(c), c_ref), f"K={K} tile={tile}"


def test_k_not_a_multiple_of_8_is_refused():
    ctx = make_ctx(world_size=2, rank=0)
    for K in (100, 12, 4):
        with pytest.raises(tl.TileLinkError) as e:
            tl.tl_query_workspace(ctx, tl.TL_OP_AG_GEMM, [256, 128, K])
        assert e.value.status == tl.TL_ERR_UNSUPPORTED_SHAPE
    tl.tl_ctx_destroy(ctx)
