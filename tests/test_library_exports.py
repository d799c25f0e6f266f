"""The C-ABI library loads and exports every symbol the public header declares (no GPU calls)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tilelink_mi355.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tl_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib_path = os.path.join(ROOT, "paper_2503_20313_amd", "libtilelink_mi355.so")
    assert os.path.exists(lib_path), "build the library first (__graft_entry__.build())"
    lib = ctypes.CDLL(lib_path)
    names = declared_functions()
    assert "tl_ag_gemm" in names and "tl_gemm_rs" in names and len(names) >= 9
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"
    lib.tl_version.restype = ctypes.c_char_p
    assert b"gfx950" in lib.tl_version()


def test_binding_struct_matches_header_field_order():
    import paper_2503_20313_amd as tl
    text = open(os.path.join(ROOT, "include", "tilelink_mi355.h")).read()
    body = text[text.index("typedef struct tl_config {"):text.index("} tl_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in re.findall(r"(?:int|unsigned)\s+([^;]+);", body):
        fields += [f.strip() for f in decl.split(",")]
    assert fields == [f[0] for f in tl.tl_config._fields_]


def test_pack_gate_up_layout():
    """Column 64t + j of the packed matrix is gate column 32t + j for j < 32 and up column 32t + j - 32 otherwise."""
    import numpy as np
    import torch
    import paper_2503_20313_amd as tl
    K, F = 5, 96
    g = np.arange(K * F, dtype=np.int32).reshape(K, F)
    u = -1 - g
    p = tl.pack_gate_up(g, u)
    assert p.shape == (K, 2 * F) and p.flags["C_CONTIGUOUS"]
    for c in range(2 * F):
        t, j = divmod(c, 64)
        want = g[:, 32 * t + j] if j < 32 else u[:, 32 * t + j - 32]
        assert np.array_equal(p[:, c], want)
    pt = tl.pack_gate_up(torch.from_numpy(g), torch.from_numpy(u))
    assert torch.equal(pt, torch.from_numpy(p)) and pt.is_contiguous()
    import pytest
    with pytest.raises(ValueError):
        tl.pack_gate_up(g[:, :40], u[:, :40])


def test_bench_refuses_more_than_one_gpu():
    """One GPU's share is all this build covers: bench.py says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "--gpus must be 1" in r.stderr and r.stdout.strip() == ""
