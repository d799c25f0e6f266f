"""Plain CPU definitions of the five overlapped operators (test infrastructure only).

Overlap changes *when* tiles are computed, never *what* is computed, so each
operator below is the plain definition of its result written out with numpy in
float64: an explicit gather (concatenate), one matrix product, an explicit
sum over ranks, explicit top-k routing, explicit softmax attention.  The only
roundings are the ones the data types of the layer force: every tensor that
exists in memory in the real layer is bfloat16 (round to nearest even).

bf16 tensors are numpy uint16 bit patterns.  Functions return both the rounded
bf16 result and the unrounded float64 one.

Operator definitions follow the paper's "Communication and Intra-Layer
Parallelism" section (tensor-parallel FFN = AllGather+GEMM then
GEMM+ReduceScatter; sequence-parallel attention = AllGather of K/V then local
attention), its "Kernel Design" section (GEMM+RS, AG+MoE, AG-KV+attention) and
the MoE paragraph of its evaluation (AG+Gather+GroupGEMM and
GroupGEMM+Scatter+TopkReduce+RS).
"""
from __future__ import annotations

import numpy as np

from .bf16 import round_to_bf16, widen


# ---------------------------------------------------------------------------
# AllGather + GEMM   (tensor-parallel FFN, first half)
# ---------------------------------------------------------------------------

def all_gather_rows(shards):
    """Explicit AllGather along the first axis: rank order concatenation."""
    return np.concatenate([np.asarray(s) for s in shards], axis=0)


def ag_gemm(a_shards, b):
    """C = AllGather_M(A_shards) . B with B given as [K, N].

    Returns (gathered A bits [M,K], C float64 [M,N], C bf16 bits [M,N])."""
    a = all_gather_rows(a_shards)
    c = widen(a) @ widen(b)
    return a, c, round_to_bf16(c)


def push_all_gather(shards):
    """AllGather in push mode, all ranks at once (paper: data primitives, push mode: every producer writes its local
    data to all other ranks): rank r's shard lands at rows [r*m, (r+1)*m) of every rank's gathered matrix.
    Returns the R gathered matrices (bf16 bits)."""
    R, m = len(shards), shards[0].shape[0]
    gathered = [np.zeros((R * m,) + shards[0].shape[1:], dtype=shards[0].dtype) for _ in range(R)]
    for r in range(R):                 # rank r pushes (and keeps its own rows)
        for q in range(R):
            gathered[q][r * m:(r + 1) * m] = shards[r]
    return gathered


def ag_gemm_push(a_shards, b, rank):
    """AllGather + GEMM of rank `rank` in push mode: its gathered matrix and product as in ag_gemm, plus what it
    delivers: slots[q] = the copy of its shard that lands in peer q's gathered matrix (None for q = rank).

    Returns (gathered A bits, C float64, C bf16 bits, slots)."""
    a, c, c_bits = ag_gemm(a_shards, b)
    slots = [None if q == rank else np.array(a_shards[rank], copy=True) for q in range(len(a_shards))]
    return a, c, c_bits, slots


def act_mul(gate, up, act):
    """The activation layer between the two halves of the MLP layer (paper,
    evaluation, "MLP Layer": SiLUMul or GeLUMul), elementwise in float64:
    "silu": gate * sigmoid(gate) * up;  "gelu": gate * Phi(gate) * up with Phi
    the standard normal distribution function."""
    from scipy.special import erf
    gate = np.asarray(gate, dtype=np.float64)
    up = np.asarray(up, dtype=np.float64)
    if act == "silu":
        return gate / (1.0 + np.exp(-gate)) * up
    if act == "gelu":
        return gate * 0.5 * (1.0 + erf(gate / np.sqrt(2.0))) * up
    raise ValueError(act)


def ag_gemm_act_mul(a_shards, w_gate, w_up, act):
    """Y = act(A . W_gate) * (A . W_up) with A = AllGather_M(A_shards), both
    weights [K, F].  The activation is applied to the unrounded products (a
    kernel that folds it into the GEMM never stores them), so Y is rounded once.

    Returns (gathered A bits [M,K], Y float64 [M,F], Y bf16 bits [M,F])."""
    a = all_gather_rows(a_shards)
    y = act_mul(widen(a) @ widen(w_gate), widen(a) @ widen(w_up), act)
    return a, y, round_to_bf16(y)


# ---------------------------------------------------------------------------
# GEMM + ReduceScatter   (tensor-parallel FFN, second half)
# ---------------------------------------------------------------------------

def reduce_scatter_segment(own_segment_bits, peer_segments, rank):
    """Sum over ranks q = 0..R-1 of the rows of partial q that belong to `rank`.
    `peer_segments[q]` is [M/R, N] bf16 (entry `rank` is ignored, the local
    partial's own rows are `own_segment_bits`)."""
    total = np.zeros(own_segment_bits.shape, dtype=np.float64)
    for q in range(len(peer_segments)):
        total += widen(own_segment_bits if q == rank else peer_segments[q])
    return total


def gemm_rs(a, b, peer_segments, rank):
    """P = bf16(A . B) (the local partial, stored as a tensor of the layer's
    dtype); out = bf16( sum_q P_q[rows of segment `rank`] ).

    Returns (P bits [M,N], out float64 [M/R,N], out bf16 bits)."""
    R = len(peer_segments)
    p = round_to_bf16(widen(a) @ widen(b))
    seg = p.shape[0] // R
    own = p[rank * seg:(rank + 1) * seg]
    out = reduce_scatter_segment(own, peer_segments, rank)
    return p, out, round_to_bf16(out)


def ring_hop(own_rows, incoming):
    """One hop of the ring ReduceScatter (paper: kernel design, GEMM + ring ReduceScatter: local reduction, then the
    partial result is passed to the previous rank): the running sum that leaves a rank is its own partial rows plus
    what it received, as a tensor of the layer's dtype; the rank that starts a chain (incoming is None) passes its
    own rows on unchanged.  bf16 bits in, bf16 bits out."""
    if incoming is None:
        return np.array(own_rows, copy=True)
    return round_to_bf16(widen(own_rows) + widen(incoming))


def ring_rs_rank(p, ring_recv, rank):
    """What rank `rank` of a ring ReduceScatter does with its partial result p [M,N] (bf16 bits).  The running sum of
    segment q travels rank q-1 -> q-2 -> ... -> q (mod R): ring_recv[q] is what rank+1 handed on for segment q (None
    for q = rank+1, whose chain starts here).

    Returns (passed: list of R, entry q = the running sum handed to rank-1 for segment q, None for q = rank;
             out bf16 bits [M/R,N] = the finished sum of segment `rank`)."""
    R = len(ring_recv)
    seg = p.shape[0] // R
    passed, out = [None] * R, None
    for step in range(R):                      # chain order: segment rank+1 first, the own segment last
        q = (rank + 1 + step) % R
        v = ring_hop(p[q * seg:(q + 1) * seg], None if step == 0 else ring_recv[q])
        if q == rank:
            out = v
        else:
            passed[q] = v
    return passed, out


def ring_reduce_scatter(partials):
    """All R ranks of the ring at once (for checking the one-rank function against the definition of a
    ReduceScatter): partials[r] = rank r's [M,N] partial result.  Returns (outs: entry r = rank r's [M/R,N] result,
    recv: recv[r][q] = what rank r received for segment q)."""
    R = len(partials)
    seg = partials[0].shape[0] // R
    recv = [[None] * R for _ in range(R)]
    outs = [None] * R
    for step in range(R):
        for r in range(R):
            q = (r + 1 + step) % R             # the segment rank r handles at this step
            v = ring_hop(partials[r][q * seg:(q + 1) * seg], recv[r][q])
            if step == R - 1:
                outs[r] = v
            else:
                recv[(r - 1) % R][q] = v
    return outs, recv


def gemm_ring_rs(a, b, ring_recv, rank):
    """P = bf16(A . B), then this rank's part of the ring ReduceScatter of P (ring_rs_rank).

    Returns (P bits [M,N], passed, out bf16 bits)."""
    p = round_to_bf16(widen(a) @ widen(b))
    passed, out = ring_rs_rank(p, ring_recv, rank)
    return p, passed, out


# ---------------------------------------------------------------------------
# MoE routing -> dynamic mapping tables
# ---------------------------------------------------------------------------

def moe_route(logits, topk, renormalize=True):
    """Top-k routing of every token.

    The k experts of a token are those with the k largest gate logits (softmax
    is monotonic, so this equals the k largest probabilities); equal logits go
    to the lower expert index; experts are listed by descending logit.  The
    routing weight is the softmax probability over all E experts, divided by
    the sum over the selected k when `renormalize`.

    Returns (topk_ids [T,k] int32, topk_w [T,k] float64)."""
    logits = np.asarray(logits, dtype=np.float32)
    T, E = logits.shape
    ids = np.zeros((T, topk), dtype=np.int32)
    for t in range(T):
        row = logits[t]
        # sort by (-logit, index): python's sort is stable and exact on float32 values
        order = sorted(range(E), key=lambda e: (-float(row[e]), e))
        ids[t] = order[:topk]
    x = logits.astype(np.float64)
    x = x - x.max(axis=1, keepdims=True)
    p = np.exp(x)
    p /= p.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, ids.astype(np.int64), axis=1)
    if renormalize:
        w = w / w.sum(axis=1, keepdims=True)
    return ids, w


def moe_sort_rows(topk_ids, E):
    """Routed row (t, j) has id t*k + j and expert topk_ids[t, j].  Rows are put
    in expert order, ascending row id inside an expert (a stable counting sort).

    Returns (expert_count [E], expert_offset [E+1], sorted_row [T*k]) int32."""
    T, k = topk_ids.shape
    flat = topk_ids.reshape(-1)
    count = np.zeros(E, dtype=np.int32)
    for e in flat:
        count[e] += 1
    offset = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        offset[e + 1] = offset[e] + count[e]
    cursor = offset[:-1].copy()
    sorted_row = np.zeros(T * k, dtype=np.int32)
    for row in range(T * k):
        e = flat[row]
        sorted_row[cursor[e]] = row
        cursor[e] += 1
    return count, offset, sorted_row


def moe_tile_tables(expert_offset, sorted_row, T, topk, R, C, Tm):
    """Dynamic mapping tables, one row of 8 int32 per grouped-GEMM row tile:
    (f_S_low, f_S_high, expert, chan_mask_lo, chan_mask_hi, f_R_lo, f_R_hi, 0).

    Expert e owns ceil(count[e]/Tm) tiles over its run of sorted rows; the last
    one is short.  chan_mask has bit (rank*C + local channel) set for every
    AllGather channel that holds a token of the tile (bits 0..31 in _lo, 32..63
    in _hi); f_R_lo..f_R_hi is the span of source ranks."""
    E = len(expert_offset) - 1
    tokens_per_rank = T // R
    tokens_per_channel = tokens_per_rank // C
    rows = []
    for e in range(E):
        lo = int(expert_offset[e])
        end = int(expert_offset[e + 1])
        while lo < end:
            hi = min(lo + Tm, end)
            mask = 0
            ranks = []
            for s in range(lo, hi):
                token = int(sorted_row[s]) // topk
                mask |= 1 << (token // tokens_per_channel)
                ranks.append(token // tokens_per_rank)
            lo32 = mask & 0xFFFFFFFF
            hi32 = (mask >> 32) & 0xFFFFFFFF
            to_i32 = lambda v: v - (1 << 32) if v >= (1 << 31) else v
            rows.append((lo, hi, e, to_i32(lo32), to_i32(hi32), min(ranks), max(ranks), 0))
            lo = hi
    return np.array(rows, dtype=np.int32).reshape(-1, 8)


# ---------------------------------------------------------------------------
# MoE part 1: AllGather + Gather + GroupGEMM
# ---------------------------------------------------------------------------

def moe_ag_gather_gemm(x_shards, w1, sorted_row, expert_offset, topk):
    """Y1[s, :] = bf16( X[token(s), :] . W1[expert(s)] ) for every sorted row s,
    X = AllGather of the token shards, token(s) = sorted_row[s] // topk.

    Returns (gathered X bits, Y1 float64 [T*k, I], Y1 bf16 bits)."""
    x = all_gather_rows(x_shards)
    xf = widen(x)
    E, H, I = w1.shape
    y = np.zeros((len(sorted_row), I), dtype=np.float64)
    for e in range(E):
        lo, hi = int(expert_offset[e]), int(expert_offset[e + 1])
        if hi > lo:
            tokens = np.asarray(sorted_row[lo:hi], dtype=np.int64) // topk
            y[lo:hi] = xf[tokens] @ widen(w1[e])
    return x, y, round_to_bf16(y)


def moe_ag_gather_gemm_act_mul(x_shards, w_gate, w_up, sorted_row, expert_offset, topk, act):
    """MoE part 1 with the expert FFN's activation: Y1[s, :] = act(x . Wgate[e]) * (x . Wup[e]) for x = the token of
    sorted row s and e = its expert; both weights [E, H, F]; the activation (act_mul) is applied to the unrounded
    products, one rounding.

    Returns (gathered X bits, Y1 float64 [T*k, F], Y1 bf16 bits)."""
    x = all_gather_rows(x_shards)
    xf = widen(x)
    E, H, F = w_gate.shape
    y = np.zeros((len(sorted_row), F), dtype=np.float64)
    for e in range(E):
        lo, hi = int(expert_offset[e]), int(expert_offset[e + 1])
        if hi > lo:
            tokens = np.asarray(sorted_row[lo:hi], dtype=np.int64) // topk
            y[lo:hi] = act_mul(xf[tokens] @ widen(w_gate[e]), xf[tokens] @ widen(w_up[e]), act)
    return x, y, round_to_bf16(y)


# ---------------------------------------------------------------------------
# MoE part 2: GroupGEMM + Scatter + TopkReduce + ReduceScatter
# ---------------------------------------------------------------------------

def moe_gemm_scatter_rs(x2, w2, sorted_row, expert_offset, topk_w, peer_segments, rank):
    """Z[s,:] = bf16( w[row(s)] * (X2[s,:] . W2[expert(s)]) ), stored at
    scatter_buf[sorted_row[s], :] (row id = token*k + slot);
    partial[t,:] = bf16( sum_j scatter_buf[t*k + j, :] );
    out = bf16( sum over ranks of the partial rows of segment `rank` ).

    Returns (scatter_buf bits [T*k,H], partial bits [T,H], out float64, out bits)."""
    E, I, H = w2.shape
    n_rows = len(sorted_row)
    T, k = topk_w.shape
    w_flat = np.asarray(topk_w, dtype=np.float64).reshape(-1)
    x2f = widen(x2)
    scatter = np.zeros((n_rows, H), dtype=np.uint16)
    for e in range(E):
        lo, hi = int(expert_offset[e]), int(expert_offset[e + 1])
        if hi > lo:
            rows = np.asarray(sorted_row[lo:hi], dtype=np.int64)
            z = (x2f[lo:hi] @ widen(w2[e])) * w_flat[rows][:, None]
            scatter[rows] = round_to_bf16(z)
    partial_f = widen(scatter).reshape(T, k, H).sum(axis=1)
    partial = round_to_bf16(partial_f)
    R = len(peer_segments)
    seg = T // R
    out = reduce_scatter_segment(partial[rank * seg:(rank + 1) * seg], peer_segments, rank)
    return scatter, partial, out, round_to_bf16(out)


# ---------------------------------------------------------------------------
# Sequence-parallel attention: AllGather K/V + softmax attention
# ---------------------------------------------------------------------------

def sp_ag_attention(q, k_shards, v_shards, rank, causal=True, scale=None, heads=None, rows=None):
    """O[i,h,:] = sum_j softmax_j(scale * <Q[i,h,:], K[j,h,:]>) V[j,h,:], with K, V
    the row-concatenation of all ranks' shards and, when causal, j restricted to
    j <= g where g = rank * S/R + i is the query's global position.

    `heads` / `rows` restrict the computation to some heads / local query rows
    (for sampled checks at full size).  Returns (K bits, V bits, O float64
    [len(rows), len(heads), D], O bf16 bits)."""
    k = all_gather_rows(k_shards)
    v = all_gather_rows(v_shards)
    S_loc, Hd, D = q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    heads = list(range(Hd)) if heads is None else list(heads)
    rows = np.arange(S_loc) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((len(rows), len(heads), D), dtype=np.float64)
    g = rank * S_loc + rows                                    # global positions
    for hi, h in enumerate(heads):
        qh = widen(q[rows, h, :])
        kh = widen(k[:, h, :])
        vh = widen(v[:, h, :])
        for blk in range(0, len(rows), 256):
            sl = slice(blk, min(blk + 256, len(rows)))
            s = (qh[sl] @ kh.T) * scale
            if causal:
                s = np.where(np.arange(k.shape[0])[None, :] <= g[sl][:, None], s, -np.inf)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            out[sl, hi, :] = (p @ vh) / p.sum(axis=1, keepdims=True)
    return k, v, out, round_to_bf16(out)


# ---------------------------------------------------------------------------
# Error measures used by the parity tests
# ---------------------------------------------------------------------------

def rel_frobenius(got_bits, ref_bits):
    g, r = widen(got_bits), widen(ref_bits)
    return float(np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300))


def max_abs_over_max_ref(got_bits, ref_bits):
    g, r = widen(got_bits), widen(ref_bits)
    return float(np.max(np.abs(g - r)) / max(np.max(np.abs(r)), 1e-300))
