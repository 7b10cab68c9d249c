"""What the compiler made of the hot kernels (no GPU needed: hipcc cross-compiles gfx950): none of them may spill
registers to scratch memory, and each has to keep the occupancy its launch bounds were chosen for."""
import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2205_09707_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# kernel (prefix of the mangled name's readable part) -> (source file, most vector registers, most LDS bytes)
KERNELS = {
    "scq_mfma_kernelILi2E": ("k_scq.hip", 128, 40 << 10),          # four waves per SIMD, four workgroups per CU
    "scq_mfma_kernelILi1E": ("k_scq.hip", 128, 40 << 10),
    "stage1_tail_kernelILi2ELb0E": ("k_scq.hip", 128, 64 << 10),   # 1024 threads: 128 registers at most
    "stage1_tail_kernelILi8ELb0E": ("k_scq.hip", 128, 64 << 10),
    "stage1_tail_kernelILi2ELb1E": ("k_scq.hip", 128, 64 << 10),   # ... also with the re-evaluations in double
    "stage1_tail_kernelILi8ELb1E": ("k_scq.hip", 128, 64 << 10),
    "scq16_kernelILi2ELb1E": ("k_scq16.hip", 256, 40 << 10),       # two waves per SIMD, two to four workgroups per CU
    "s2_invert_kernelILi11EjE": ("k_stage2.hip", 168, 53 << 10),   # 2048 passages per workgroup, three workgroups (of four waves) per CU
    "s2_invert_kernelILi11EyE": ("k_stage2.hip", 168, 53 << 10),
    "s2_invert_kernelILi13EjE": ("k_stage2.hip", 128, 80 << 10),   # 8192 passages, 1024 threads, 32-bit sets: two per CU
    "s2_invert_kernelILi13EyE": ("k_stage2.hip", 128, 100 << 10),  # ... 64-bit sets: one per CU
    "s2_union_wide_kernel": ("k_stage2.hip", 128, 80 << 10),       # two workgroups of 1024 threads per CU
    "s2_stream_kernel": ("k_stage2.hip", 128, 40 << 10),
    "ci_list_kernelILb0E": ("k_ci.hip", 96, 8 << 10),              # five waves per SIMD; wave-private LDS areas
    "decompress_maxsim_kernelILi2ELb0ELb0E": ("k_stage4.hip", 128, 32 << 10),   # four waves per SIMD (query operands in LDS)
    "decompress_maxsim_kernelILi1ELb0ELb0E": ("k_stage4.hip", 128, 32 << 10),
    "decompress_maxsim_kernelILi2ELb0ELb1E": ("k_stage4.hip", 128, 32 << 10),   # ... with unit-length reconstruction
    "sel_sort_kernelILi512E": ("k_select.hip", 64, 0),             # dynamic LDS only
    "sel2_filter_kernel": ("k_select.hip", 64, 8 << 10),
    "encode_residuals_kernelILi2E": ("k_build.hip", 64, 0),
    "ivb_rank_kernel": ("k_build.hip", 64, 0),
    "ivb_sort_short_kernel": ("k_build.hip", 64, 32 << 10),      # a 2048-entry LDS area per wave
    "ivb_sort_long_kernel": ("k_build.hip", 128, 130 << 10),     # a bitmap of 2^20 passage ids: one workgroup (16 waves) per CU
}


def _assembly(src, out):
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fno-gpu-rdc", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "--cuda-device-only", "-S",
           os.path.join(CSRC, src), "-o", out]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return open(out).read()


def _metadata(text):
    """name -> dict of the integer fields of each kernel's metadata record"""
    out = {}
    for rec in text.split("  - .agpr_count:")[1:]:
        name = re.search(r"\.name:\s+(\S+)", rec).group(1)
        f = {k: int(v) for k, v in re.findall(r"\.(\w+):\s+(\d+)\n", rec)}
        f["agpr_count"] = int(rec.split("\n", 1)[0])
        out[name] = f
    return out


@pytest.mark.skipif(not (os.path.exists(HIPCC) or shutil.which("hipcc")), reason="hipcc not installed")
def test_hot_kernels_do_not_spill(tmp_path):
    files = sorted({v[0] for v in KERNELS.values()})
    with ThreadPoolExecutor(max_workers=len(files)) as ex:
        texts = dict(zip(files, ex.map(lambda f: _assembly(f, str(tmp_path / (f[:-4] + ".s"))), files)))
    meta = {f: _metadata(t) for f, t in texts.items()}
    for key, (src, max_vgpr, max_lds) in KERNELS.items():
        hits = [(n, m) for n, m in meta[src].items() if key in n]
        assert len(hits) == 1, f"{key}: {len(hits)} kernels match in {src}"
        name, m = hits[0]
        assert m["vgpr_spill_count"] == 0 and m["private_segment_fixed_size"] == 0, f"{name} spills: {m}"
        assert m["vgpr_count"] + m["agpr_count"] <= max_vgpr, f"{name}: {m['vgpr_count']} + {m['agpr_count']} registers"
        assert m["group_segment_fixed_size"] <= max_lds, f"{name}: {m['group_segment_fixed_size']} bytes of LDS"
