"""Pins of the oracle's activation layer and gated AG+GEMM (paper, evaluation, "MLP Layer": SiLUMul / GeLUMul between
AllGather+GEMM and GEMM+ReduceScatter), and of the host-side weight packing of the gated entry point."""
import math

import numpy as np
import pytest

import tl_workloads as wl
from oracle import ops
from oracle.bf16 import round_to_bf16, widen


def test_activation_values_and_identities():
    # textbook values: sigmoid(1) = 0.7310585786300049, Phi(1) = 0.8413447460685429
    assert ops.act_mul(1.0, 2.0, "silu") == pytest.approx(2 * 0.7310585786300049, rel=1e-15)
    assert ops.act_mul(1.0, 2.0, "gelu") == pytest.approx(2 * 0.8413447460685429, rel=1e-15)
    assert ops.act_mul(0.0, 5.0, "silu") == 0.0 and ops.act_mul(0.0, 5.0, "gelu") == 0.0
    x = np.linspace(-9, 9, 181)
    for act in ("silu", "gelu"):
        f = ops.act_mul(x, 1.0, act)
        assert np.allclose(f - ops.act_mul(-x, 1.0, act), x, rtol=0, atol=1e-14)     # x*s(x) + x*s(-x) = x for s = sigmoid, Phi
        assert np.allclose(ops.act_mul(x, 3.0, act), 3.0 * f, rtol=1e-15)            # linear in `up`
        assert abs(ops.act_mul(40.0, 1.0, act) - 40.0) < 1e-12 and abs(ops.act_mul(-40.0, 1.0, act)) < 1e-12
    # the two differ (a swapped name would show): silu(2) = 1.7615941559557649, gelu(2) = 2*Phi(2) = 1.9544997361036416
    assert ops.act_mul(2.0, 1.0, "silu") == pytest.approx(1.7615941559557649, rel=1e-14)
    assert ops.act_mul(2.0, 1.0, "gelu") == pytest.approx(2 * 0.5 * (1 + math.erf(2 / math.sqrt(2))), rel=1e-14)
    assert ops.act_mul(2.0, 1.0, "gelu") == pytest.approx(1.9544997361036416, rel=1e-14)
    # gate and up are not interchangeable
    assert ops.act_mul(1.0, 2.0, "silu") != ops.act_mul(2.0, 1.0, "silu")


def test_gated_moe_part1_is_the_composition():
    """The gated grouped GEMM equals act_mul of the two plain grouped GEMMs (which have pins of their own), and one
    sorted row recomputed straight from the definition."""
    w = wl.moe_inputs(64, 32, 32, 4, 2, 2, 0, config_id=36)
    w_up = w["w1_up"]
    ids, _ = ops.moe_route(w["logits"], 2)[:2]
    _, off, srow = ops.moe_sort_rows(ids, 4)
    x, y, y_bits = ops.moe_ag_gather_gemm_act_mul(w["x_shards"], w["w1"], w_up, srow, off, 2, "silu")
    _, g, _ = ops.moe_ag_gather_gemm(w["x_shards"], w["w1"], srow, off, 2)
    _, u, _ = ops.moe_ag_gather_gemm(w["x_shards"], w_up, srow, off, 2)
    assert np.array_equal(y, ops.act_mul(g, u, "silu")) and np.array_equal(y_bits, round_to_bf16(y))
    s = 37
    e = int(np.searchsorted(np.asarray(off), s, side="right") - 1)
    xrow = widen(x)[int(srow[s]) // 2]
    for f in (0, 13, 31):
        gg = float(xrow @ widen(w["w1"][e])[:, f])
        uu = float(xrow @ widen(w_up[e])[:, f])
        assert y[s, f] == pytest.approx(gg / (1 + math.exp(-gg)) * uu, rel=1e-12, abs=1e-15)


@pytest.mark.parametrize("act", ["silu", "gelu"])
def test_gated_ag_gemm_is_the_composition(act):
    w = wl.ag_gemm_gated_inputs(64, 32, 48, 4, config_id=31)
    a, y, y_bits = ops.ag_gemm_act_mul(w["a_shards"], w["w_gate"], w["w_up"], act)
    assert np.array_equal(a, np.concatenate(w["a_shards"]))
    # brute force on a few entries, straight from the definition
    A, G, U = widen(a), widen(w["w_gate"]), widen(w["w_up"])
    for (i, f) in [(0, 0), (17, 5), (63, 31), (40, 16)]:
        g = sum(A[i, k] * G[k, f] for k in range(48))
        u = sum(A[i, k] * U[k, f] for k in range(48))
        s = 1 / (1 + math.exp(-g)) if act == "silu" else 0.5 * (1 + math.erf(g / math.sqrt(2)))
        assert y[i, f] == pytest.approx(g * s * u, rel=1e-12, abs=1e-15)
    assert np.array_equal(y_bits, round_to_bf16(y))
    # with up = a matrix that makes A.W_up == 1 the result is act(A.W_gate) alone: not checked here (A is random); instead
    # the two plain products recombine to the same thing
    _, g_full, _ = ops.ag_gemm(w["a_shards"], w["w_gate"])
    _, u_full, _ = ops.ag_gemm(w["a_shards"], w["w_up"])
    assert np.array_equal(y, ops.act_mul(g_full, u_full, act))
