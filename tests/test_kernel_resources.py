"""Compiler-reported resources of the search kernels (hipcc cross-compiles without a GPU): no register
spills, no scratch memory, and every single-mode kernel leaves room for at least two wavefronts per SIMD.
A change that pushes one template instance over 256 registers halves its wavefronts per CU without
failing any parity test; this one notices."""
import concurrent.futures
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2308_15136_amd", "csrc")


def _hipcc():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def _resources(src, tmp):
    out = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                          "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, src),
                          "-o", os.path.join(tmp, src + ".o")], capture_output=True, text=True, check=True).stderr
    kernels, cur = {}, None
    for line in out.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = kernels.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+) \[-Rpass", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return kernels


@pytest.mark.skipif(not os.path.exists(_hipcc()), reason="hipcc not found")
def test_search_kernels_fit_their_registers(tmp_path):
    sources = ["search_kernels_f32.hip", "search_kernels_f16.hip", "search_kernels_u8.hip", "exact_filter.hip"]
    with concurrent.futures.ThreadPoolExecutor(len(sources)) as pool:
        results = list(pool.map(lambda s: _resources(s, str(tmp_path)), sources))
    seen = 0
    for src, kernels in zip(sources, results):
        assert kernels, f"no resource remarks for {src}"
        for name, r in kernels.items():
            if "search_" not in name and "mfma_tile" not in name and "rerank" not in name:
                continue
            seen += 1
            assert r.get("VGPRs Spill", 0) == 0 and r.get("ScratchSize", 0) == 0, f"{name}: {r}"
            if "search_single" in name or "mfma_tile" in name:      # throughput kernels; the multi mode trades
                assert r.get("Occupancy", 0) >= 2, f"{name}: {r}"   # wavefronts for rows in flight on purpose
    assert seen >= 3 * (24 + 12 + 8) + 3
