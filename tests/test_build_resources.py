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


def _check(kernels, pattern, expect_count, spill_free=True):
    hit = {k: v for k, v in kernels.items() if re.search(pattern, k)}
    assert len(hit) == expect_count, (pattern, sorted(kernels))
    for name, res in hit.items():
        if spill_free:
            assert res["VGPRs Spill"] == 0 and res["SGPRs Spill"] == 0 and res["ScratchSize [bytes/lane]"] == 0, (name, res)
        assert res["Occupancy [waves/SIMD]"] >= 2, (name, res)
    return hit


def _scratch_in_inner_loops(src, pattern):
    """For every kernel of `src` whose mangled name matches: the scratch instructions that lie inside an innermost loop
    (from the block annotations of the compiler's assembly listing).  A spill outside the loops costs a few instructions
    once; one inside a key loop costs a scratch round trip per tile."""
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "x.s")
        r = subprocess.run(["hipcc", *B.FLAGS, "-S", "--cuda-device-only", os.path.join(B.CSRC, src), "-o", out],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(out).read().splitlines()
    found, cur, inner, in_inner = {}, None, set(), False
    for line in text:
        m = re.match(r"^(_Z\w+):", line)
        if m:
            cur = m.group(1) if re.search(pattern, m.group(1)) else None
            if cur:
                found[cur] = []
            inner, in_inner = set(), False
            continue
        if cur is None:
            continue
        m = re.match(r"^(\.LBB\d+_\d+):(.*)", line)
        if m:
            label, note = m.group(1), m.group(2)
            if "Inner Loop Header" in note:
                inner.add(label.lstrip("."))
                in_inner = True
            else:
                h = re.search(r"in Loop: Header=(BB\d+_\d+)", note)
                in_inner = bool(h) and ("L" + h.group(1)) in {"L" + x.lstrip("L") for x in inner}
            continue
        if re.match(r"^; %bb\.\d+:", line):
            h = re.search(r"in Loop: Header=(BB\d+_\d+)", line)
            in_inner = bool(h) and ("L" + h.group(1)) in {"L" + x.lstrip("L") for x in inner}
            continue
        if in_inner and "scratch_" in line:
            found[cur].append(line.strip())
    return found


def test_forward_kernels_do_not_spill():
    k = _resources("fwd.hip")
    # fwd_kernel<D, TRAIN, CAUSAL, DUMP, PQ, VARLEN>: every production variant (DUMP = false), d = 64 and 128, the three block
    # forms of phi(P); the bf16 P-tilde of the mixed recipe (inference only); the per-sequence lengths of the paged forward
    _check(k, r"fwd_kernelILi(64|128)ELb[01]ELb0ELb0ELi[012]ELb0E", 12)
    _check(k, r"fwd_kernelILi(64|128)ELb0ELb0ELb0ELi3ELb0E", 2)
    _check(k, r"fwd_kernelILi(64|128)ELb0ELb0ELb0ELi0ELb1E", 2)
    # Causal variants: a workgroup takes two query tiles one after the other, and the compiler parks a few values that only
    # the set-up and the wind-down of a tile use (the lane number, two constants) in scratch across the key loop.  What must
    # not happen is a scratch access inside the key loop.
    causal = r"fwd_kernelILi(64|128)ELb[01]ELb1ELb0ELi[0123]ELb[01]E"      # 12 + 2 (bf16 P-tilde) + 2 (per-sequence lengths)
    hit = _check(k, causal, 16, spill_free=False)
    # (scalar registers parked in lanes of a vector register cost no memory access: up to 16 of them, mostly the MX variants,
    #  which carry the addresses of two more operand arrays)
    assert all(v["VGPRs Spill"] <= 8 and v["SGPRs Spill"] <= 16 for v in hit.values()), hit
    inner = _scratch_in_inner_loops("fwd.hip", causal)
    assert len(inner) == 16 and all(not v for v in inner.values()), {n: v for n, v in inner.items() if v}


def test_backward_kernels_do_not_spill():
    k = _resources("bwd.hip")
    _check(k, r"bwd_dq_kernelILi(64|128)ELb[01]ELb[01]ELi[48]E", 16)    # <D, CAUSAL, scores on the FP4 instruction (MX), waves>
    # bwd_dkdv_kernel<D, CAUSAL, COUNT, PQ>: the measurement (COUNT) and ablation (PQ = 0) variants are exempt
    _check(k, r"bwd_dkdv_kernelILi(64|128)ELb[01]ELb0ELi[123]ELi[48]E", 24)   # 12 of 4 waves, 12 of 8


def test_decode_kernels_do_not_spill():
    k = _resources("decode.hip")
    hit = _check(k, r"decode_kernelILi(64|128)ELb[01]E", 4, spill_free=False)
    # no scratch memory; scalar registers parked in vector lanes are tolerated (the kernel takes twenty arguments)
    assert all(v["VGPRs Spill"] == 0 and v["ScratchSize [bytes/lane]"] == 0 for v in hit.values()), hit


def test_mx_forward_kernels_do_not_spill():
    k = _resources("mx.hip")
    # fwd_mx_kernel<D, CAUSAL, FP8PV, KVM>: 8 contiguous variants, the 4 paged and the 4 block-sparse ones (FP4 only)
    _check(k, r"fwd_mx_kernelILi(64|128)ELb[01]ELb[01]ELi[012]E", 16)
    # fwd_mx_decode_kernel<D, CAUSAL, NP = 1>: two workgroups per CU
    _check(k, r"fwd_mx_decode_kernelILi(64|128)ELb[01]ELi1E", 4)
