"""Register budget of the kernels, read from the compiler's own metadata (no GPU): a wave of a communication side kernel
must fit on a SIMD beside two waves of the matrix kernel it serves (512 vector registers per SIMD lane, allocated in
blocks of 8), no side kernel may take more than 56, no matrix kernel that runs beside one more than 232, and nothing
may spill vector registers."""
import os
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2503_20313_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def kernel_registers(source):
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-S", "--cuda-device-only", "-o", out, os.path.join(CSRC, source)]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-2000:]
        text = open(out).read()
    regs = {}
    for m in re.finditer(r"\.name:\s+(\S+)\n(.*?)\.vgpr_count:\s+(\d+)\n\s+\.vgpr_spill_count:\s+(\d+)", text, re.S):
        scratch = re.search(r"\.private_segment_fixed_size:\s+(\d+)", m.group(2))
        sgpr_spill = re.search(r"\.sgpr_spill_count:\s+(\d+)", m.group(2))
        regs[m.group(1)] = dict(vgpr=int(m.group(3)), spill=int(m.group(4)), scratch=int(scratch.group(1)) if scratch else 0,
                                sgpr_spill=int(sgpr_spill.group(1)) if sgpr_spill else 0)
    return regs


def test_register_budget():
    with ThreadPoolExecutor(3) as ex:
        parts = list(ex.map(kernel_registers, ["tl_dense.hip", "tl_moe.hip", "tl_attention.hip"]))
    regs = {k: v for part in parts for k, v in part.items()}
    assert len(regs) >= 15, sorted(regs)
    def find(pattern):
        hits = [k for k in regs if re.search(pattern, k)]
        assert hits, pattern
        return hits

    def alloc(k):
        return -(-regs[k]["vgpr"] // 8) * 8

    side = find(r"ag_producer_kernel|rs_consumer_kernel|kv_producer_kernel|moe_ag_producer_kernel|moe_reduce_kernel")
    assert len(side) == 5, side
    for k in side:
        assert regs[k]["vgpr"] <= 56, (k, regs[k])
    # the matrix kernels of the default launch configurations (256x256 tile; attention) with the side kernel beside them
    pairs = [(r"ag_gemm_kernel.*Li256ELi256E", r"ag_producer_kernel"), (r"gemm_rs_kernel.*Li256ELi256E", r"rs_consumer_kernel"),
             (r"moe_gemm_scatter_kernel.*Li256ELi256E", r"moe_reduce_kernel"), (r"sp_attention_kernel", r"kv_producer_kernel")]
    for mat, sd in pairs:
        for m in find(mat):
            assert regs[m]["vgpr"] <= 232, (m, regs[m])
            for s_ in find(sd):
                assert 2 * alloc(m) + alloc(s_) <= 512, (m, regs[m]["vgpr"], s_, regs[s_]["vgpr"])
    for k, r in regs.items():
        assert r["spill"] == 0, (k, r)
        assert r["scratch"] <= 128, (k, r)       # a few SGPR spill slots at most, no arrays in scratch memory
