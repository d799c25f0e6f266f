"""Register budget of the kernels, read from the compiler's own metadata (no GPU): the communication side kernels must
fit into the 48 vector registers that two waves of a matrix kernel leave on a SIMD (512 - 2 * 232), the matrix kernels
that run beside them must stay at or below 232, and nothing may spill."""
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
    side = [k for k in regs if re.search(r"ag_producer_kernel|rs_consumer_kernel|kv_producer_kernel|moe_ag_producer_kernel|moe_reduce_kernel", k)]
    assert len(side) == 5, side
    for k in side:
        assert regs[k]["vgpr"] <= 48, (k, regs[k])
    # the matrix kernels of the default launch configurations (256x256 tile; attention), all of which run beside a side kernel
    beside = [k for k in regs if ("TileCfgILi256ELi256E" in k and re.search(r"ag_gemm_kernel|gemm_rs_kernel|moe_gemm_scatter_kernel", k)) or "sp_attention_kernel" in k]
    assert len(beside) >= 5, beside
    for k in beside:
        assert regs[k]["vgpr"] <= 232, (k, regs[k])
    for k, r in regs.items():
        assert r["spill"] == 0, (k, r)
        assert r["scratch"] <= 128, (k, r)       # a few SGPR spill slots at most, no arrays in scratch memory
