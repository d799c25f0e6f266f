"""Seeded synthetic inputs for the overlapped tensor-parallel operators.

This module only draws random numbers and stores them as bfloat16 / float32 /
int arrays.  It contains none of the operators' arithmetic: no GEMM, no
reduction, no routing, no attention, no tile mapping.  Both the CPU oracle's
tests and the GPU tests/benchmarks take their inputs from here, so the two
sides always see identical bits.

bfloat16 tensors are numpy ``uint16`` arrays holding the bit patterns (numpy has
no bfloat16 dtype).  The shapes follow the paper's benchmark table (MLP-5,
MoE-5, Attn-1 at 32k, all reduced to one rank's share of a TP=8 layer); the
value distributions are the ones the task's configurations name.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 250320313


def _rng(config_id: int, tensor_id: int, shard_id: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([BASE_SEED, config_id, tensor_id, shard_id])))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> bfloat16 bit patterns (round to nearest, ties to even).

    Used only to store freshly drawn samples as bf16 inputs."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def normal_bf16(shape, std, config_id, tensor_id, shard_id=0) -> np.ndarray:
    g = _rng(config_id, tensor_id, shard_id)
    x = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return to_bf16_bits(x)


def uniform_bf16(shape, lo, hi, config_id, tensor_id, shard_id=0) -> np.ndarray:
    g = _rng(config_id, tensor_id, shard_id)
    x = g.random(size=shape, dtype=np.float32) * np.float32(hi - lo) + np.float32(lo)
    return to_bf16_bits(x)


def normal_f32(shape, std, config_id, tensor_id, shard_id=0) -> np.ndarray:
    g = _rng(config_id, tensor_id, shard_id)
    x = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


# ----------------------------------------------------------------------------
# Workload recipes.  Each returns a dict of arrays plus the integer dimensions.
# ----------------------------------------------------------------------------

def ag_gemm_inputs(M, N, K, world, config_id=2, a_dist="normal", b_std=0.02):
    """A sharded along M into `world` shards of [M/world, K]; B is [K, N]."""
    assert M % world == 0
    ms = M // world
    if a_dist == "normal":
        shards = [normal_bf16((ms, K), 1.0, config_id, 0, q) for q in range(world)]
    else:
        shards = [uniform_bf16((ms, K), -1.0, 1.0, config_id, 0, q) for q in range(world)]
    b = normal_bf16((K, N), b_std, config_id, 1)
    return {"a_shards": shards, "b": b, "M": M, "N": N, "K": K, "world": world}


def ag_gemm_gated_inputs(M, F, K, world, config_id=6, b_std=0.02):
    """A sharded along M as in ag_gemm_inputs; gate and up projection weights, each [K, F]."""
    w = ag_gemm_inputs(M, F, K, world, config_id=config_id, b_std=b_std)
    return {"a_shards": w["a_shards"], "w_gate": w["b"], "w_up": normal_bf16((K, F), b_std, config_id, 2),
            "M": M, "F": F, "K": K, "world": world}


def gemm_rs_inputs(M, N, K, world, rank, config_id=3, b_std=0.02, peer_std=None):
    """Local A [M,K], B [K,N]; for every peer q != rank the rows of its partial
    product that fall in this rank's output segment, [M/world, N] bf16.

    A real peer's partial is the product of its own K-slice; here it is drawn
    N(0, sigma) with sigma = sqrt(K)*b_std so that it has the same scale."""
    assert M % world == 0
    a = normal_bf16((M, K), 1.0, config_id, 0)
    b = normal_bf16((K, N), b_std, config_id, 1)
    if peer_std is None:
        peer_std = float(np.sqrt(K)) * b_std
    seg = M // world
    peers = [None if q == rank else normal_bf16((seg, N), peer_std, config_id, 2, q) for q in range(world)]
    return {"a": a, "b": b, "peer_segments": peers, "M": M, "N": N, "K": K, "world": world, "rank": rank}


def gemm_ring_rs_inputs(M, N, K, world, rank, config_id=7, b_std=0.02):
    """Local A [M,K], B [K,N]; for every segment q != rank+1 the running sum [M/world, N] bf16 that rank+1 hands on
    in a ring ReduceScatter.  The chain of segment q starts at rank q-1 and comes down the ranks, so what arrives
    here already holds (q-1-rank) mod world partial products: drawn N(0, sigma) with sigma = sqrt(that count * K) * b_std."""
    assert M % world == 0
    a = normal_bf16((M, K), 1.0, config_id, 0)
    b = normal_bf16((K, N), b_std, config_id, 1)
    seg = M // world
    recv = []
    for q in range(world):
        count = (q - 1 - rank) % world
        recv.append(None if count == 0 else normal_bf16((seg, N), float(np.sqrt(count * K)) * b_std, config_id, 2, q))
    return {"a": a, "b": b, "ring_recv": recv, "M": M, "N": N, "K": K, "world": world, "rank": rank}


def moe_inputs(T, H, I, E, topk, world, rank, config_id=4, w_std=0.02):
    """Token shards [T/world,H], gate logits [T,E] fp32, expert weights W1 [E,H,I]
    (and a second one of the same shape, the "up" projection of a gated expert FFN),
    W2 [E,I,H], an independently seeded second-half input X2 [T*topk, I] and the
    peers' partial-output slices [T/world, H]."""
    assert T % world == 0
    ts = T // world
    x_shards = [normal_bf16((ts, H), 1.0, config_id, 0, q) for q in range(world)]
    logits = normal_f32((T, E), 1.0, config_id, 1)
    w1 = normal_bf16((E, H, I), w_std, config_id, 2)
    w2 = normal_bf16((E, I, H), w_std, config_id, 3)
    x2 = normal_bf16((T * topk, I), 1.0, config_id, 4)
    peer_std = float(np.sqrt(I)) * w_std
    peers = [None if q == rank else normal_bf16((ts, H), peer_std, config_id, 5, q) for q in range(world)]
    w1_up = normal_bf16((E, H, I), w_std, config_id, 6)
    return {"x_shards": x_shards, "logits": logits, "w1": w1, "w1_up": w1_up, "w2": w2, "x2": x2,
            "peer_segments": peers,
            "T": T, "H": H, "I": I, "E": E, "topk": topk, "world": world, "rank": rank}


def sp_attention_inputs(S, heads, head_dim, world, config_id=5):
    """Q of one rank [S/world, heads, D] is drawn per rank by the caller through
    `shard_id`; K and V shards [S/world, heads, D] for every rank."""
    assert S % world == 0
    ss = S // world
    q_shards = [normal_bf16((ss, heads, head_dim), 1.0, config_id, 0, q) for q in range(world)]
    k_shards = [normal_bf16((ss, heads, head_dim), 1.0, config_id, 1, q) for q in range(world)]
    v_shards = [normal_bf16((ss, heads, head_dim), 1.0, config_id, 2, q) for q in range(world)]
    return {"q_shards": q_shards, "k_shards": k_shards, "v_shards": v_shards,
            "S": S, "heads": heads, "head_dim": head_dim, "world": world}


# The named configurations (index = position in the benchmark's config list, 1-based).
CONFIGS = {
    1: dict(op="ag_gemm", M=256, N=512, K=512, world=2, a_dist="uniform"),
    2: dict(op="ag_gemm", M=8192, N=3584, K=8192, world=8, a_dist="normal"),
    3: dict(op="gemm_rs", M=8192, N=8192, K=3584, world=8),
    4: dict(op="moe", T=8192, H=4096, I=1792, E=32, topk=2, world=8),
    5: dict(op="sp_attention", S=32768, heads=32, head_dim=128, world=8),
}
