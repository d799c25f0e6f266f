"""Pins for the oracle's ring ReduceScatter (paper: kernel design, GEMM + ring ReduceScatter).

The ring is tied to the definition of a ReduceScatter (segment r of the sum over ranks ends at rank r): exactly on
integer data, within the roundings of the R-1 hops on random data; the one-rank function is tied to the all-rank
simulation, and the roles of the segments (where a chain starts, where it ends, which incoming buffer is unused) to
direct statements about them.
"""
import numpy as np
import pytest

import tl_workloads as wl
from oracle import ops
from oracle.bf16 import round_to_bf16, widen


def int_partials(R, M, N, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    return [round_to_bf16(rng.integers(-8, 9, size=(M, N)).astype(np.float64)) for _ in range(R)]


@pytest.mark.parametrize("R", [1, 2, 3, 4, 8])
def test_ring_equals_reduce_scatter_exactly_on_integers(R):
    """Small integers: every running sum is an integer below 256, which bf16 holds exactly, so the ring must give the
    plain sum over ranks of segment r at rank r, bit for bit."""
    M, N = 4 * R, 8
    parts = int_partials(R, M, N, 700 + R)
    outs, _ = ops.ring_reduce_scatter(parts)
    total = sum(widen(p) for p in parts)
    seg = M // R
    for r in range(R):
        assert np.array_equal(outs[r], round_to_bf16(total[r * seg:(r + 1) * seg]))
        assert np.array_equal(widen(outs[r]), total[r * seg:(r + 1) * seg])


def test_ring_on_random_data_is_within_the_hops_roundings():
    R, M, N = 8, 64, 32
    parts = [wl.normal_bf16((M, N), 1.0, 71, 0, r) for r in range(R)]
    outs, _ = ops.ring_reduce_scatter(parts)
    total = sum(widen(p) for p in parts)
    seg = M // R
    some_differ = False
    for r in range(R):
        ref = total[r * seg:(r + 1) * seg]
        err = np.linalg.norm(widen(outs[r]) - ref) / np.linalg.norm(ref)
        assert err <= (R - 1) * 2.0 ** -9                         # one rounding (half an ulp of 2^-8) per hop
        some_differ |= not np.array_equal(outs[r], round_to_bf16(ref))
    assert some_differ       # the hops do round: a ring that summed in one go would not differ from the plain sum


@pytest.mark.parametrize("R", [2, 5, 8])
def test_one_rank_function_matches_the_all_rank_ring(R):
    M, N = 8 * R, 16
    parts = [wl.normal_bf16((M, N), 1.0, 72, 0, r) for r in range(R)]
    outs, recv = ops.ring_reduce_scatter(parts)
    for r in range(R):
        passed, out = ops.ring_rs_rank(parts[r], recv[r], r)
        assert np.array_equal(out, outs[r])
        assert passed[r] is None
        for q in range(R):
            if q != r:
                assert np.array_equal(passed[q], recv[(r - 1) % R][q])      # what leaves rank r arrives at rank r-1
        assert recv[r][(r + 1) % R] is None                                # nothing arrives for the chain that starts at r


def test_roles_of_the_segments():
    R, rank, M, N = 4, 2, 16, 8
    seg = M // R
    p = wl.normal_bf16((M, N), 1.0, 73, 0)
    recv = [wl.normal_bf16((seg, N), 1.0, 73, 1, q) for q in range(R)]
    passed, out = ops.ring_rs_rank(p, recv, rank)
    start = (rank + 1) % R
    # the chain of segment rank+1 starts here: the partial rows go on unchanged, whatever sits in ring_recv[rank+1]
    assert np.array_equal(passed[start], p[start * seg:(start + 1) * seg])
    junk = list(recv)
    junk[start] = np.full((seg, N), 0x7FC0, dtype=np.uint16)
    passed2, out2 = ops.ring_rs_rank(p, junk, rank)
    assert np.array_equal(out2, out) and all(np.array_equal(a, b) for a, b in zip(passed2, passed) if a is not None)
    # every other segment: own rows + incoming, rounded once; the own segment ends in `out`
    for q in range(R):
        if q == start:
            continue
        want = round_to_bf16(widen(p[q * seg:(q + 1) * seg]) + widen(recv[q]))
        assert np.array_equal(out if q == rank else passed[q], want)
    # one element by hand
    i, j, q = 1, 3, 0
    s = float(widen(p[q * seg + i:q * seg + i + 1, j:j + 1])[0, 0]) + float(widen(recv[q][i:i + 1, j:j + 1])[0, 0])
    assert passed[q][i, j] == round_to_bf16(np.array([s]))[0]


def test_gemm_ring_rs_uses_the_rounded_product():
    w = wl.gemm_ring_rs_inputs(32, 16, 64, 4, 1, config_id=74)
    assert w["ring_recv"][2] is None and all(w["ring_recv"][q] is not None for q in (0, 1, 3))
    p, passed, out = ops.gemm_ring_rs(w["a"], w["b"], w["ring_recv"], 1)
    p_ref, _, _ = ops.gemm_rs(w["a"], w["b"], [np.zeros((8, 16), np.uint16)] * 4, 1)   # the pinned GEMM + rounding
    assert np.array_equal(p, p_ref)
    passed_ref, out_ref = ops.ring_rs_rank(p, w["ring_recv"], 1)
    assert np.array_equal(out, out_ref) and np.array_equal(passed[0], passed_ref[0])
    # scale of the incoming running sums: (q-1-rank) mod R partial products of std sqrt(K)*0.02 each
    for q, count in ((3, 1), (0, 2), (1, 3)):
        assert np.std(widen(w["ring_recv"][q])) == pytest.approx(np.sqrt(count * 64) * 0.02, rel=0.25)
