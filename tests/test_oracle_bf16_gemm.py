"""Pins for the oracle's bf16 rounding, AllGather+GEMM and GEMM+ReduceScatter.

Each check ties the oracle to something other than itself: hand-computed bit
patterns, an exhaustive round trip, a library conversion routine, exact integer
arithmetic with python ints, closed forms and the invariants of the collectives.
"""
from fractions import Fraction

import numpy as np
import torch

import tl_workloads as wl
from oracle import ops
from oracle.bf16 import round_to_bf16, widen


def bits_to_torch(bits):
    return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)


# ----------------------------------------------------------------------------- bf16

def test_bf16_hand_values():
    # 1.0, -2.0, 0.5, largest finite, smallest normal
    x = np.array([1.0, -2.0, 0.5, float.fromhex("0x1.fep127"), 2.0 ** -126, 0.0])
    assert list(round_to_bf16(x)) == [0x3F80, 0xC000, 0x3F00, 0x7F7F, 0x0080, 0x0000]
    # ties go to the even significand: 1+2^-8 is halfway between 0x3F80 and 0x3F81 -> 0x3F80;
    # 1+3*2^-8 is halfway between 0x3F81 and 0x3F82 -> 0x3F82
    assert list(round_to_bf16(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8]))) == [0x3F80, 0x3F82]
    # just above / below the tie
    assert list(round_to_bf16(np.array([1 + 2.0 ** -8 + 2.0 ** -30, 1 + 3 * 2.0 ** -8 - 2.0 ** -30]))) == [0x3F81, 0x3F81]
    # overflow to infinity, and a value that would double-round wrongly through float32:
    # 1 + 2^-8 + 2^-40 must go up (float32 would first drop the 2^-40 and then tie to even, down)
    assert list(round_to_bf16(np.array([3.4e38, -3.4e38, 1 + 2.0 ** -8 + 2.0 ** -40]))) == [0x7F80, 0xFF80, 0x3F81]


def test_bf16_exhaustive_round_trip():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = widen(bits)
    keep = ~np.isnan(f)
    assert np.array_equal(round_to_bf16(f[keep]), bits[keep])


def test_bf16_matches_library_conversion_on_float32_values():
    g = np.random.default_rng(7)
    x = (g.standard_normal(200000) * np.exp(g.uniform(-30, 30, 200000))).astype(np.float32)
    x = np.concatenate([x, np.array([1e-40, -1e-40, 2.0 ** -133, 3 * 2.0 ** -134], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(round_to_bf16(x.astype(np.float64)), want)
    # the input generator's own conversion agrees too (it is separate code)
    assert np.array_equal(wl.to_bf16_bits(x), want)


# ----------------------------------------------------------------------------- AllGather + GEMM

def small_int_bf16(shape, seed, lo=-4, hi=5):
    g = np.random.default_rng(seed)
    vals = g.integers(lo, hi, size=shape).astype(np.float64)
    return round_to_bf16(vals), vals.astype(np.int64)


def test_gather_is_concatenation():
    w = wl.ag_gemm_inputs(64, 16, 32, 4, config_id=91)
    a, _, _ = ops.ag_gemm(w["a_shards"], w["b"])
    assert a.shape == (64, 32)
    for q in range(4):
        assert np.array_equal(a[q * 16:(q + 1) * 16], w["a_shards"][q])


def test_ag_gemm_exact_integers_non_square():
    # small integers: every product and sum is exact, so the result is fixed with no tolerance;
    # non-square M,N,K catches any transposed operand or swapped index
    shards, ints = zip(*[small_int_bf16((5, 7), 100 + q) for q in range(3)])
    b_bits, b_int = small_int_bf16((7, 11), 200)
    _, c, c_bits = ops.ag_gemm(list(shards), b_bits)
    a_int = np.concatenate(ints, axis=0)
    want = np.zeros((15, 11), dtype=np.int64)
    for i in range(15):
        for j in range(11):
            for k in range(7):
                want[i, j] += int(a_int[i, k]) * int(b_int[k, j])
    assert np.array_equal(c, want.astype(np.float64))
    assert np.array_equal(widen(c_bits), want.astype(np.float64))   # |values| < 256: exact in bf16


def test_ag_gemm_brute_force_rationals():
    w = wl.ag_gemm_inputs(8, 6, 10, 2, config_id=92)
    _, c, c_bits = ops.ag_gemm(w["a_shards"], w["b"])
    a = np.concatenate(w["a_shards"])
    af, bf = widen(a), widen(w["b"])
    for i in range(8):
        for j in range(6):
            exact = sum(Fraction(float(af[i, k])) * Fraction(float(bf[k, j])) for k in range(10))
            assert abs(Fraction(float(c[i, j])) - exact) <= abs(exact) * Fraction(1, 2 ** 45) + Fraction(1, 2 ** 80)
            # the bf16 result is one of the two bf16 neighbours of the exact value and the nearer one
            got = Fraction(float(widen(c_bits[i:i + 1, j:j + 1])[0, 0]))
            ulp = Fraction(2) ** (int(np.floor(np.log2(max(abs(float(exact)), 1e-300)))) - 7)
            assert abs(got - exact) <= ulp / 2


def test_ag_gemm_identity_and_ones():
    w = wl.ag_gemm_inputs(32, 24, 24, 4, config_id=93)
    eye = round_to_bf16(np.eye(24))
    a, _, c_bits = ops.ag_gemm(w["a_shards"], eye)
    assert np.array_equal(c_bits, a)                       # B = I  =>  C == gathered A, bit for bit
    ones = [round_to_bf16(np.ones((8, 24))) for _ in range(4)]
    _, c, _ = ops.ag_gemm(ones, w["b"])
    colsum = widen(w["b"]).sum(axis=0)
    assert np.allclose(c, np.broadcast_to(colsum, (32, 24)), rtol=1e-13, atol=1e-13)


def test_ag_gemm_matches_library_matmul():
    w = wl.ag_gemm_inputs(256, 512, 512, 2, config_id=1, a_dist="uniform")
    _, c, c_bits = ops.ag_gemm(w["a_shards"], w["b"])
    at = torch.cat([bits_to_torch(s) for s in w["a_shards"]]).double()
    ct = at @ bits_to_torch(w["b"]).double()
    assert torch.allclose(torch.from_numpy(c), ct, rtol=1e-12, atol=1e-12)
    # bf16 rounding of the float64 product: torch rounds float32 -> bf16; go through float32 only
    # where that is exact enough not to matter (differences allowed on <0.01% of entries, 1 ulp)
    lib = ct.float().to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.mean(lib != c_bits) < 1e-4


# ----------------------------------------------------------------------------- GEMM + ReduceScatter

def test_gemm_rs_peers_zero_and_peers_equal():
    R, rank = 4, 2
    w = wl.gemm_rs_inputs(32, 16, 24, R, rank, config_id=94)
    zeros = [None if q == rank else np.zeros((8, 16), dtype=np.uint16) for q in range(R)]
    p, _, out_bits = ops.gemm_rs(w["a"], w["b"], zeros, rank)
    assert np.array_equal(out_bits, p[rank * 8:(rank + 1) * 8])          # nothing to add: own rows, bit exact
    same = [None if q == rank else p[rank * 8:(rank + 1) * 8].copy() for q in range(R)]
    _, out, out_bits = ops.gemm_rs(w["a"], w["b"], same, rank)
    assert np.array_equal(widen(out_bits), 4.0 * widen(p[rank * 8:(rank + 1) * 8]))   # power-of-two scaling is exact


def test_gemm_rs_real_peers_sum_to_full_product():
    # split a full GEMM along K over R ranks; reduce-scatter of the partials == full product
    R, M, N, Kfull = 4, 32, 20, 64
    a_full = wl.normal_bf16((M, Kfull), 1.0, 95, 0)
    b_full = wl.normal_bf16((Kfull, N), 0.05, 95, 1)
    ks = Kfull // R
    partial = [round_to_bf16(widen(a_full[:, q * ks:(q + 1) * ks]) @ widen(b_full[q * ks:(q + 1) * ks])) for q in range(R)]
    seg = M // R
    outs = []
    for r in range(R):
        peers = [None if q == r else partial[q][r * seg:(r + 1) * seg] for q in range(R)]
        p, out, _ = ops.gemm_rs(a_full[:, r * ks:(r + 1) * ks], b_full[r * ks:(r + 1) * ks], peers, r)
        assert np.array_equal(p, partial[r])
        outs.append(out)
    full = widen(a_full) @ widen(b_full)
    got = np.concatenate(outs)
    # only the bf16 rounding of the R partials separates the two: R * 2^-9 relative to the partial scale
    assert np.max(np.abs(got - full)) <= R * 2.0 ** -8 * np.max(np.abs(widen(np.stack(partial))))
    assert np.linalg.norm(got - full) / np.linalg.norm(full) < 5e-3


def test_reduce_scatter_exact_integers_and_rank_selectivity():
    R = 3
    segs = [round_to_bf16(np.full((2, 4), float(q + 1))) for q in range(R)]
    for rank in range(R):
        own = round_to_bf16(np.full((2, 4), 10.0))
        peers = [None if q == rank else segs[q] for q in range(R)]
        out = ops.reduce_scatter_segment(own, peers, rank)
        assert np.all(out == 10.0 + sum(q + 1 for q in range(R) if q != rank))


def test_push_all_gather_gives_every_rank_the_gathered_matrix():
    """Push mode delivers the same matrix as the definition of AllGather (rows of rank r at r*m), at every rank, and a
    rank's deliveries are exact copies of its shard."""
    R = 4
    shards = [wl.normal_bf16((6, 8), 1.0, 93, 0, r) for r in range(R)]
    want = ops.all_gather_rows(shards)
    for g in ops.push_all_gather(shards):
        assert np.array_equal(g, want)
    assert np.array_equal(want[2 * 6:3 * 6], shards[2]) and not np.array_equal(want[0:6], shards[2])
    w = wl.ag_gemm_inputs(32, 16, 64, 4, config_id=94)
    a, c, c_bits, slots = ops.ag_gemm_push(w["a_shards"], w["b"], 1)
    a2, c2, c_bits2 = ops.ag_gemm(w["a_shards"], w["b"])
    assert np.array_equal(a, a2) and np.array_equal(c_bits, c_bits2)
    assert slots[1] is None and all(np.array_equal(slots[q], w["a_shards"][1]) for q in (0, 2, 3))
