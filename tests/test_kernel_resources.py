"""What the compiler made of the kernels (no GPU needed: hipcc cross-compiles for gfx950 and
reports each kernel's registers, LDS and scratch).  The row-copy kernels must keep the chunks a
lane has in flight in registers: a local array of them was once promoted to LDS, 16 KB per
workgroup, which cost the hit gather a fifth of its rate; and no kernel may spill to scratch."""
import os
import re
import subprocess
import tempfile

import pytest


def resource_usage(source):
    from paper_2112_08541_amd import buildlib
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc is not installed")
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [hipcc, *buildlib.HIPCC_FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c",
               os.path.join(buildlib.CSRC, source), "-o", os.path.join(tmp, "x.o")]
        p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert p.returncode == 0, p.stdout[-2000:]
    kernels, name = {}, None
    for line in p.stdout.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            kernels[name] = {}
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+)", line)
        if m and name:
            kernels[name][m.group(1).strip()] = int(m.group(2))
    return kernels


def test_row_copy_kernels_keep_their_chunks_in_registers():
    kernels = resource_usage("bgl_cache.hip")
    copies = {k: v for k, v in kernels.items()
              if re.search(r"k_gather_hits|k_fetch_miss|k_fetch_rows|k_insert_rows|k_assemble_rows", k)}
    assert len(copies) >= 4 * (1 + 2 + 4 + 1 + 1)   # four row widths of each variant
    for name, use in copies.items():
        assert use["LDS Size"] == 0, (name, use)
        assert use["Occupancy"] == 8, (name, use)
    for name, use in kernels.items():
        assert use["ScratchSize"] == 0, (name, use)
        if "k_assemble_pre" in name:                 # its per-wavefront lists of (position, slot): 4 x 64 x 8 bytes
            assert use["LDS Size"] == 2048, (name, use)
            continue
        assert use["LDS Size"] <= 1024, (name, use)  # scan scratch only; the sampler's hash table lives in bgl_sample.hip


def test_sampling_kernels_use_the_lds_they_declare():
    kernels = resource_usage("bgl_sample.hip")
    for name, use in kernels.items():
        assert use["ScratchSize"] == 0, (name, use)
        if "k_sample_insert" in name:
            # dedup table 2 x 512 x 8 B + its 2 x 512 x 4 B of entry indices + scan scratch
            assert use["LDS Size"] == 8192 + 4096 + 32, (name, use)
