"""Helpers for the GPU parity tests: upload/download of bf16 bit patterns and a harness that
owns the device buffers of one operator call."""
import numpy as np
import torch

import paper_2503_20313_amd as tl
from oracle import ops

REL_FRO_TOL = 5e-3      # relative Frobenius error vs the oracle's bf16 output
MAX_ABS_TOL = 1e-2      # max |got - ref| / max |ref|
POISON = 0x7FC0         # bf16 quiet NaN


def dev():
    return torch.device("cuda:0")


def up(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev())


def down(t):
    return t.cpu().numpy().view(np.uint16)


def poison(shape):
    return torch.full(shape, POISON, dtype=torch.int16, device=dev()).view(torch.int16) if False else \
        torch.from_numpy(np.full(shape, POISON, dtype=np.uint16).view(np.int16)).to(dev())


def assert_close_bf16(got_bits, ref_bits, what=""):
    g = ops.widen(got_bits) if hasattr(ops, "widen") else None
    from oracle.bf16 import widen
    g, r = widen(got_bits), widen(ref_bits)
    assert not np.isnan(g).any(), f"{what}: NaN in the GPU result (a tile was read before it was ready, or never written)"
    rel = float(np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300))
    mx = float(np.max(np.abs(g - r)) / max(np.max(np.abs(r)), 1e-300))
    assert rel <= REL_FRO_TOL and mx <= MAX_ABS_TOL, f"{what}: rel_fro={rel:.3e} max_abs/max_ref={mx:.3e}"
    return rel, mx


def make_ctx(**kw):
    base = dict(world_size=1, rank=0, channels_per_rank=1, comm_mode=tl.TL_COMM_WAVES, tile_order=tl.TL_ORDER_RING,
                xcd_swizzle=1, spin_timeout_us=5_000_000)
    base.update(kw)
    return tl.tl_ctx_create(**base)
