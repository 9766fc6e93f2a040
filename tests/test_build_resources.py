"""The attention kernels run at 2 waves per SIMD with all 256 registers in use: a register spill in
a hot loop costs a scratch round trip per tile (and, because vector-memory loads return in order, a
wait for the tile prefetch in flight).  This test compiles the kernels with the compiler's resource
remarks and fails if a production kernel spills or loses its occupancy.  CPU only: hipcc cross-compiles."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

from paper_2603_00040_amd import build as B

pytestmark = pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")


def _resources(src):
    with tempfile.TemporaryDirectory() as tmp:
        r = subprocess.run(["hipcc", *B.FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c",
                            os.path.join(B.CSRC, src), "-o", os.path.join(tmp, "x.o")],
                           capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    out, cur = {}, None
    for line in r.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+(VGPRs Spill|SGPRs Spill|Occupancy \[waves/SIMD\]|ScratchSize \[bytes/lane\]): (\d+)", line)
        if m and cur is not None:
            cur[m.group(1)] = int(m.group(2))
    return out


def _check(kernels, pattern, expect_count):
    hit = {k: v for k, v in kernels.items() if re.search(pattern, k)}
    assert len(hit) == expect_count, (pattern, sorted(kernels))
    for name, res in hit.items():
        assert res["VGPRs Spill"] == 0 and res["SGPRs Spill"] == 0 and res["ScratchSize [bytes/lane]"] == 0, (name, res)
        assert res["Occupancy [waves/SIMD]"] >= 2, (name, res)


def test_forward_kernels_do_not_spill():
    k = _resources("fwd.hip")
    # fwd_kernel<D, TRAIN, CAUSAL, DUMP, PQ>: every production variant (DUMP = false), d = 64 and 128, the three forms of phi(P)
    _check(k, r"fwd_kernelILi(64|128)ELb[01]ELb[01]ELb0ELi[012]E", 24)


def test_backward_kernels_do_not_spill():
    k = _resources("bwd.hip")
    _check(k, r"bwd_dq_kernelILi(64|128)ELb[01]E", 4)
    # bwd_dkdv_kernel<D, CAUSAL, COUNT, PQ>: the measurement (COUNT) and ablation (PQ = 0) variants are exempt
    _check(k, r"bwd_dkdv_kernelILi(64|128)ELb[01]ELb0ELi[123]E", 12)


def test_mx_forward_kernels_do_not_spill():
    k = _resources("mx.hip")
    # fwd_mx_kernel<D, CAUSAL, FP8PV, KVM>: 8 contiguous variants, the 4 paged and the 4 block-sparse ones (FP4 only)
    _check(k, r"fwd_mx_kernelILi(64|128)ELb[01]ELb[01]ELi[012]E", 16)
    # fwd_mx_decode_kernel<D, CAUSAL, NP = 1>: two workgroups per CU
    _check(k, r"fwd_mx_decode_kernelILi(64|128)ELb[01]ELi1E", 4)
