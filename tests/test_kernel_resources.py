"""Register budgets of the two hot kernels, read from the compiler's own resource report (no GPU needed).

The verify attention runs two workgroups per compute unit, i.e. 256 registers per wavefront, and its streaming loop
uses every one of them: a change anywhere in the kernel that makes the register allocator spill puts scratch
accesses into that loop (measured: 2-3 % of a launch).  The GEMM's hot instances likewise must not touch scratch.
"""
import os
import re
import subprocess
import tempfile

import pytest

import paper_2508_18588_amd as hs

CSRC = os.path.join(os.path.dirname(os.path.abspath(hs.__file__)), "csrc")
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(hs.__file__)))


def resource_report(source):
    """{mangled kernel name: {field: int}} from -Rpass-analysis=kernel-resource-usage (device code only)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in hs.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory(prefix="hs_res_") as tmp:
        p = subprocess.run([hipcc] + flags + ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "--cuda-device-only",
                                              "-c", os.path.join(CSRC, source), "-o", os.path.join(tmp, "dev.o"),
                                              "-Rpass-analysis=kernel-resource-usage"],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert p.returncode == 0, p.stdout[-2000:]
    report, cur = {}, None
    for line in p.stdout.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = report.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z /\[\]]+?):\s+(\d+)\s+\[-Rpass", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return report


def test_verify_attention_keeps_two_workgroups_per_compute_unit_without_scratch():
    rep = resource_report("hs_attention.hip")
    kernels = {k: v for k, v in rep.items() if "attn_verify_mfma" in k}
    assert len(kernels) == 2, sorted(rep)                      # head_dim 128 and 64
    for name, r in kernels.items():
        assert r["ScratchSize [bytes/lane]"] == 0 and r["VGPRs Spill"] == 0, (name, r)
        assert r["Occupancy [waves/SIMD]"] >= 2, (name, r)
        assert r["LDS Size [bytes/block]"] <= 80 * 1024, (name, r)


def test_hot_gemm_instances_use_no_scratch():
    rep = resource_report("hs_gemm_stream.hip")
    # <EPI, PARTIAL, NU, MT, SA, SW> of a 7B-shape speculative step: gate/up, down, QKV and O, LM head (row maximum);
    # and the same at 128 rows (the one-token steps)
    hot = ["ILi2ELb0ELi5ELi3ELi2ELi3EE", "ILi0ELb1ELi4ELi3ELi2ELi4EE", "ILi0ELb1ELi2ELi3ELi2ELi6EE",
           "ILi3ELb0ELi5ELi3ELi2ELi3EE", "ILi2ELb0ELi5ELi2ELi2ELi4EE", "ILi0ELb1ELi4ELi2ELi2ELi5EE",
           "ILi0ELb1ELi2ELi2ELi2ELi8EE", "ILi3ELb0ELi5ELi2ELi2ELi4EE"]
    for tag in hot:
        names = [k for k in rep if "hs_gemm_stream" + tag in k]
        assert len(names) == 1, (tag, sorted(rep))
        r = rep[names[0]]
        assert r["ScratchSize [bytes/lane]"] == 0 and r["VGPRs Spill"] == 0, (names[0], r)
