"""GPU parity at further shapes of the paper's benchmark table (one rank's TP=8 share each), in the launch configuration
bench.py uses (side-kernel binding, own-first order, direct push).  The dense operators are checked on a sample of
output columns (the oracle runs on those columns of B only), MoE in full, attention on sampled heads and rows."""
import numpy as np
import pytest

import paper_2503_20313_amd as tl
import tl_workloads as wl
from oracle import ops
from tests.gpu_util import assert_close_bf16
from tests.test_gpu_ag_gemm import run_ag_gemm
from tests.test_gpu_attention import check_gathered, run_attention
from tests.test_gpu_gemm_rs import run_gemm_rs
from tests.test_gpu_moe import run_part1, run_part2

pytestmark = pytest.mark.gpu
R = 8
# name -> (S, H, I) of the paper's MLP table
MLP = {"MLP-1": (8192, 4096, 11008), "MLP-2": (8192, 4096, 14336), "MLP-3": (8192, 3584, 14336), "MLP-4": (8192, 4608, 36864),
       "MLP-6": (8192, 8192, 29568)}


def sample_columns(N, n, seed):
    """n distinct columns: the first and last 8 (ragged last tile) plus random ones, sorted."""
    rng = np.random.Generator(np.random.Philox(seed))
    cols = set(range(8)) | set(range(N - 8, N)) | set(rng.choice(N, size=n, replace=False).tolist())
    return np.array(sorted(cols))


@pytest.mark.parametrize("name,rank,kc", [("MLP-1", 3, 4), ("MLP-2", 6, 4), ("MLP-3", 1, 4), ("MLP-4", 0, 1), ("MLP-6", 7, 1)])
def test_ag_gemm_mlp_shares(name, rank, kc):
    """kc = flags per AllGather channel along K as bench.py chooses them: four where one round of tiles holds the whole GEMM."""
    S, H, I = MLP[name]
    N = I // R                                       # 1376, 4608, 3696: the last two column tiles are ragged for 1376 and 3696
    w = wl.ag_gemm_inputs(S, N, H, R, config_id=60 + rank)
    hs, g, c, flags, info = run_ag_gemm(w, rank, 4, tl.TL_COMM_SIDE_KERNEL, tile_order=tl.TL_ORDER_OWN_FIRST, ag_k_chunks=kc)
    assert info["k_chunks"] == kc
    cols = sample_columns(N, 384, 600 + rank)
    a_ref, _, c_ref = ops.ag_gemm(hs, np.ascontiguousarray(w["b"][:, cols]))
    assert np.array_equal(g, a_ref)
    assert_close_bf16(c[:, cols], c_ref, f"AG+GEMM {name} share rank {rank} tile {info['tile_m']}x{info['tile_n']}")
    assert flags.tolist() == [info["expected_per_channel"]] * (R * 4 * kc)


@pytest.mark.parametrize("name,rank,direct", [("MLP-1", 5, 1), ("MLP-2", 4, 1), ("MLP-3", 0, 0), ("MLP-6", 2, 1)])
def test_gemm_rs_mlp_shares(name, rank, direct):
    S, H, I = MLP[name]
    K = I // R                                       # 1376 = 43 K steps of 32; 3696 = 115 steps and a zero-filled half step
    w = wl.gemm_rs_inputs(S, H, K, R, rank, config_id=70 + rank)
    ha, partial, push, out, flags, info = run_gemm_rs(w, tl.TL_COMM_SIDE_KERNEL, tile_order=tl.TL_ORDER_OWN_FIRST, rs_direct_push=direct)
    cols = sample_columns(H, 384, 700 + rank)
    peers = [None if p is None else np.ascontiguousarray(p[:, cols]) for p in w["peer_segments"]]
    p_ref, _, out_ref = ops.gemm_rs(ha, np.ascontiguousarray(w["b"][:, cols]), peers, rank)
    seg = S // R
    assert_close_bf16(partial[rank * seg:(rank + 1) * seg][:, cols], p_ref[rank * seg:(rank + 1) * seg], f"GEMM+RS {name} own partial")
    for q in range(R):
        if q != rank:
            assert_close_bf16(push[q][:, cols], p_ref[q * seg:(q + 1) * seg], f"GEMM+RS {name} push to {q}")
    assert_close_bf16(out[:, cols], out_ref, f"GEMM+RS {name} share rank {rank} out")
    assert not (out == 0x7FC0).any()


def test_moe_topk5_share():
    """MoE-3 of the paper's table (H=2048, I=1536, 32 experts, top-5), one rank's share of the expert FFN (I/8 = 192)."""
    w = wl.moe_inputs(8192, 2048, 192, 32, 5, R, 6, config_id=81)
    run_part1(w, 6, 2, tl.TL_COMM_SIDE_KERNEL)
    run_part2(w, tl.TL_COMM_SIDE_KERNEL, tile_order=tl.TL_ORDER_OWN_FIRST, rs_direct_push=1)


def test_moe_8_experts_share():
    """MoE-1-like: 8 experts, top-2 (2048 rows per expert: long runs of full tiles), H=2048, I/8 = 192."""
    w = wl.moe_inputs(8192, 2048, 192, 8, 2, R, 1, config_id=82)
    run_part1(w, 1, 4, tl.TL_COMM_SIDE_KERNEL)
    run_part2(w, tl.TL_COMM_SIDE_KERNEL, tile_order=tl.TL_ORDER_OWN_FIRST, rs_direct_push=1)


@pytest.mark.parametrize("S,heads,rank,causal", [(16384, 64, 5, True), (8192, 32, 2, False), (65536, 32, 7, True), (131072, 32, 6, True)])
def test_attention_other_configs(S, heads, rank, causal):
    """Attn-2 (64 heads) at 16k causal, non-causal attention at 8k, and Attn-1 at 64k and 128k (the long rows of the
    paper's table: 32 and 64 query blocks per head, shards of 8192 and 16384 keys); sampled heads and rows."""
    w = wl.sp_attention_inputs(S, heads, 128, R, config_id=90 + rank)
    res = run_attention(w, rank, causal, tl.TL_COMM_SIDE_KERNEL)
    S_loc = S // R
    rows = np.array(sorted({0, 1, 31, 32, 255, 256, 257, S_loc // 2 - 1, S_loc // 2, S_loc - 257, S_loc - 256, S_loc - 2, S_loc - 1}))
    hsel = [0, 7, heads // 2 + 1, heads - 1]
    _, _, _, o_ref = ops.sp_ag_attention(w["q_shards"][rank], w["k_shards"], w["v_shards"], rank, causal, heads=hsel, rows=rows)
    assert_close_bf16(res["o"][rows][:, hsel], o_ref, f"attention S={S} heads={heads} rank {rank} causal={causal}")
    check_gathered(w, res, rank, causal, 1)
    assert not (res["o"] == 0x7FC0).any()
