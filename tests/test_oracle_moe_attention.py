"""Pins for the oracle's MoE routing/tables, grouped GEMMs and sequence-parallel attention."""
import numpy as np
import torch

import tl_workloads as wl
from oracle import ops
from oracle.bf16 import round_to_bf16, widen


def bits_to_torch(bits):
    return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)


# ----------------------------------------------------------------------------- routing

def test_route_hand_example_with_ties():
    # token 0: logits (1, 3, 3, 0) -> tie between experts 1 and 2 goes to the lower index first
    # token 1: all equal -> experts 0, 1
    logits = np.array([[1.0, 3.0, 3.0, 0.0], [2.0, 2.0, 2.0, 2.0]], dtype=np.float32)
    ids, w = ops.moe_route(logits, 2, renormalize=True)
    assert ids.tolist() == [[1, 2], [0, 1]]
    assert np.allclose(w, [[0.5, 0.5], [0.5, 0.5]])
    ids, w = ops.moe_route(logits, 2, renormalize=False)
    z = np.exp(1.0) + 2 * np.exp(3.0) + 1.0
    assert np.allclose(w, [[np.exp(3.0) / z, np.exp(3.0) / z], [0.25, 0.25]], rtol=1e-12)
    ids, w = ops.moe_route(np.array([[0.0, 1.0, 2.0]], dtype=np.float32), 3, True)
    assert ids.tolist() == [[2, 1, 0]]                       # descending weight
    e = np.exp([2.0, 1.0, 0.0]); assert np.allclose(w[0], e / e.sum())


def test_route_against_library_topk_and_conservation():
    T, E, k = 64, 16, 3
    logits = wl.normal_f32((T, E), 1.0, 96, 0)
    ids, w = ops.moe_route(logits, k, True)
    tv, ti = torch.topk(torch.from_numpy(logits), k, dim=1)      # no ties in random data
    assert np.array_equal(ids, ti.numpy().astype(np.int32))
    p = torch.softmax(torch.from_numpy(logits).double(), dim=1).gather(1, ti)
    assert np.allclose(w, (p / p.sum(1, keepdim=True)).numpy(), rtol=1e-12)
    assert np.allclose(w.sum(axis=1), 1.0)
    count, offset, sorted_row = ops.moe_sort_rows(ids, E)
    assert count.sum() == T * k and offset[-1] == T * k
    assert sorted(sorted_row.tolist()) == list(range(T * k))            # a permutation
    for t in range(T):
        assert len(set(ids[t].tolist())) == k                           # k distinct experts
    # brute force: sort (expert, row id) pairs
    flat = ids.reshape(-1)
    brute = sorted(range(T * k), key=lambda r: (int(flat[r]), r))
    assert sorted_row.tolist() == brute
    assert np.array_equal(count, np.bincount(flat, minlength=E))


def test_route_all_experts_when_k_equals_E():
    logits = wl.normal_f32((8, 4), 1.0, 97, 0)
    ids, w = ops.moe_route(logits, 4, True)
    assert all(sorted(r) == [0, 1, 2, 3] for r in ids.tolist())
    count, _, _ = ops.moe_sort_rows(ids, 4)
    assert count.tolist() == [8, 8, 8, 8]


def test_tile_tables_hand_example():
    # T=8 tokens, k=1, R=2 ranks (4 tokens each), C=2 channels per rank (2 tokens each), Tm=3
    ids = np.array([[0], [1], [0], [0], [1], [0], [0], [1]], dtype=np.int32)
    count, offset, sorted_row = ops.moe_sort_rows(ids, 2)
    assert count.tolist() == [5, 3] and offset.tolist() == [0, 5, 8]
    assert sorted_row.tolist() == [0, 2, 3, 5, 6, 1, 4, 7]
    tab = ops.moe_tile_tables(offset, sorted_row, 8, 1, 2, 2, 3)
    # expert 0: rows [0,3) tokens 0,2,3 -> channels 0,1 ; rows [3,5) tokens 5,6 -> channels 2,3
    # expert 1: rows [5,8) tokens 1,4,7 -> channels 0,2,3
    assert tab.tolist() == [[0, 3, 0, 0b0011, 0, 0, 0, 0], [3, 5, 0, 0b1100, 0, 1, 1, 0], [5, 8, 1, 0b1101, 0, 0, 1, 0]]


def test_tile_tables_partition_rows():
    T, E, k, R, C, Tm = 256, 8, 2, 4, 2, 16
    ids, _ = ops.moe_route(wl.normal_f32((T, E), 1.0, 98, 0), k)
    count, offset, sorted_row = ops.moe_sort_rows(ids, E)
    tab = ops.moe_tile_tables(offset, sorted_row, T, k, R, C, Tm)
    pos = 0
    for lo, hi, e, mlo, mhi, rlo, rhi, _ in tab.tolist():
        assert lo == pos and lo < hi <= lo + Tm and offset[e] <= lo and hi <= offset[e + 1]
        pos = hi
        chans = {(int(sorted_row[s]) // k) // (T // (R * C)) for s in range(lo, hi)}
        assert mlo == sum(1 << c for c in chans) and mhi == 0
        assert rlo == min(c // C for c in chans) and rhi == max(c // C for c in chans)
    assert pos == T * k
    assert len(tab) == sum(-(-int(c) // Tm) for c in count)


# ----------------------------------------------------------------------------- grouped GEMMs

def test_moe_single_expert_reduces_to_dense_ops():
    R, rank, T, H, I = 2, 1, 16, 12, 10
    w = wl.moe_inputs(T, H, I, 1, 1, R, rank, config_id=99)
    ids, tw = ops.moe_route(w["logits"], 1, True)
    assert np.all(ids == 0) and np.all(tw == 1.0)
    count, offset, sorted_row = ops.moe_sort_rows(ids, 1)
    assert sorted_row.tolist() == list(range(T))
    _, y, y_bits = ops.moe_ag_gather_gemm(w["x_shards"], w["w1"], sorted_row, offset, 1)
    _, c, c_bits = ops.ag_gemm(w["x_shards"], w["w1"][0])
    assert np.array_equal(y_bits, c_bits)
    scatter, partial, out, out_bits = ops.moe_gemm_scatter_rs(w["x2"], w["w2"], sorted_row, offset, tw, w["peer_segments"], rank)
    p, out2, out2_bits = ops.gemm_rs(w["x2"], w["w2"][0], w["peer_segments"], rank)
    assert np.array_equal(scatter, p) and np.array_equal(partial, p) and np.array_equal(out_bits, out2_bits)


def test_moe_part1_rows_follow_their_token_and_expert():
    R, T, H, I, E, k = 2, 8, 6, 5, 3, 2
    w = wl.moe_inputs(T, H, I, E, k, R, 0, config_id=100)
    ids, tw = ops.moe_route(w["logits"], k)
    _, offset, sorted_row = ops.moe_sort_rows(ids, E)
    x, y, _ = ops.moe_ag_gather_gemm(w["x_shards"], w["w1"], sorted_row, offset, k)
    xf = widen(x)
    for s in range(T * k):
        row = int(sorted_row[s]); t, j = divmod(row, k); e = int(ids[t, j])
        want = [sum(xf[t, h] * widen(w["w1"][e])[h, i] for h in range(H)) for i in range(I)]
        assert np.allclose(y[s], want, rtol=1e-12, atol=1e-15)


def test_moe_part2_shared_weight_equals_dense():
    # every expert has the same W2 and the routing weights of a token sum to 1, and X2 rows of the k
    # copies of a token are identical -> the top-k reduced partial is the dense product of that row
    R, rank, T, H, I, E, k = 2, 0, 16, 8, 6, 4, 2
    w = wl.moe_inputs(T, H, I, E, k, R, rank, config_id=101)
    ids, tw = ops.moe_route(w["logits"], k, True)
    _, offset, sorted_row = ops.moe_sort_rows(ids, E)
    w2 = np.broadcast_to(w["w2"][0], w["w2"].shape).copy()
    tok_rows = wl.normal_bf16((T, I), 1.0, 101, 9)
    x2 = tok_rows[sorted_row // k]
    zeros = [None if q == rank else np.zeros((T // R, H), np.uint16) for q in range(R)]
    scatter, partial, out, _ = ops.moe_gemm_scatter_rs(x2, w2, sorted_row, offset, tw, zeros, rank)
    dense = widen(tok_rows) @ widen(w2[0])
    # two bf16 roundings (scatter rows, then the partial) separate the results
    assert np.max(np.abs(widen(partial) - dense)) <= 3 * 2.0 ** -8 * np.max(np.abs(dense))
    # scatter rows sit at (token, slot) and carry the slot's weight
    for t in range(T):
        for j in range(k):
            assert np.allclose(widen(scatter[t * k + j]), tw[t, j] * dense[t], rtol=2.0 ** -7, atol=1e-6)
    assert np.array_equal(round_to_bf16(out), partial[:T // R])


# ----------------------------------------------------------------------------- attention

def small_attn(S=32, heads=2, D=8, R=4, cfg=102):
    return wl.sp_attention_inputs(S, heads, D, R, config_id=cfg)


def test_attention_zero_query_gives_causal_running_mean():
    w = small_attn()
    R, S = 4, 32
    for rank in (0, 2, 3):
        q = np.zeros_like(w["q_shards"][rank])
        _, v, o, _ = ops.sp_ag_attention(q, w["k_shards"], w["v_shards"], rank, causal=True)
        vf = widen(v)
        for i in range(S // R):
            g = rank * (S // R) + i
            assert np.allclose(o[i], vf[:g + 1].mean(axis=0), rtol=1e-12, atol=1e-14)
        _, _, o_nc, _ = ops.sp_ag_attention(q, w["k_shards"], w["v_shards"], rank, causal=False)
        assert np.allclose(o_nc, np.broadcast_to(vf.mean(axis=0), o_nc.shape), rtol=1e-12)


def test_attention_constant_v_and_future_independence():
    w = small_attn(cfg=103)
    rank, R, S = 1, 4, 32
    const_v = [round_to_bf16(np.full(s.shape, 0.75)) for s in w["v_shards"]]
    _, _, o, _ = ops.sp_ag_attention(w["q_shards"][rank], w["k_shards"], const_v, rank)
    assert np.allclose(o, 0.75, rtol=1e-13)
    _, _, o1, _ = ops.sp_ag_attention(w["q_shards"][rank], w["k_shards"], w["v_shards"], rank)
    k2 = [s.copy() for s in w["k_shards"]]; v2 = [s.copy() for s in w["v_shards"]]
    for q in range(rank + 1, R):                     # everything after this rank's positions
        k2[q][:] = wl.normal_bf16(k2[q].shape, 3.0, 103, 7, q); v2[q][:] = wl.normal_bf16(v2[q].shape, 3.0, 103, 8, q)
    _, _, o2, _ = ops.sp_ag_attention(w["q_shards"][rank], k2, v2, rank)
    assert np.array_equal(o1, o2)
    # and inside the rank's own shard: position g sees keys <= g only
    k3 = [s.copy() for s in w["k_shards"]]
    k3[rank][5:] = 0
    _, _, o3, _ = ops.sp_ag_attention(w["q_shards"][rank], k3, w["v_shards"], rank)
    assert np.array_equal(o1[:5], o3[:5]) and not np.allclose(o1[5:], o3[5:])


def test_attention_matches_library_sdpa():
    w = small_attn(S=64, heads=3, D=16, R=4, cfg=104)
    S, R = 64, 4
    kt = torch.cat([bits_to_torch(s) for s in w["k_shards"]]).double().permute(1, 0, 2)   # [h, S, D]
    vt = torch.cat([bits_to_torch(s) for s in w["v_shards"]]).double().permute(1, 0, 2)
    for rank in range(R):
        qt = bits_to_torch(w["q_shards"][rank]).double().permute(1, 0, 2)
        g = rank * (S // R) + torch.arange(S // R)
        mask = torch.arange(S)[None, :] <= g[:, None]
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask).permute(1, 0, 2).numpy()
        _, _, o, _ = ops.sp_ag_attention(w["q_shards"][rank], w["k_shards"], w["v_shards"], rank)
        assert np.allclose(o, ref, rtol=1e-10, atol=1e-12)
        ref_nc = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt).permute(1, 0, 2).numpy()
        _, _, o_nc, _ = ops.sp_ag_attention(w["q_shards"][rank], w["k_shards"], w["v_shards"], rank, causal=False)
        assert np.allclose(o_nc, ref_nc, rtol=1e-10, atol=1e-12)
    # rank 0 equals attention over its own shard only
    qt = bits_to_torch(w["q_shards"][0]).double().permute(1, 0, 2)
    loc = torch.nn.functional.scaled_dot_product_attention(qt, kt[:, :16], vt[:, :16], is_causal=True).permute(1, 0, 2).numpy()
    _, _, o0, _ = ops.sp_ag_attention(w["q_shards"][0], w["k_shards"], w["v_shards"], 0)
    assert np.allclose(o0, loc, rtol=1e-10, atol=1e-12)
    # head / row sub-selection returns the same numbers
    _, _, osub, _ = ops.sp_ag_attention(w["q_shards"][2], w["k_shards"], w["v_shards"], 2, heads=[2, 0], rows=[3, 9])
    _, _, ofull, _ = ops.sp_ag_attention(w["q_shards"][2], w["k_shards"], w["v_shards"], 2)
    assert np.array_equal(osub, ofull[[3, 9]][:, [2, 0]])
