#!/usr/bin/env python3
"""Benchmark of the Attn-QAT hot path on one MI355X.

One step = one pass of the whole path over one batch of seeded synthetic input that is
already resident in HBM: the Q/K/V quantization passes, the training forward (Alg. 2) and
the backward (Alg. 3) for a training workload, or quantization + inference forward
(Alg. 1) for an inference workload.  Prints ONE JSON line.

FLOP convention (model FLOPs): forward 4*B*Hq*L^2*d, backward 10*B*Hq*L^2*d, halved under
a causal mask.  The roofline entry prices the dominant kernel by the MFMA work it EXECUTES
(fwd_train 6, fwd_infer 4, bwd_dq 6 times B*Hq*L^2*d; bwd_dkdv 6 + 2f, where f is the
measured fraction of 32x32 tiles whose P^F is non-zero: the dV product of the other tiles is
skipped, exactly, and is not counted) against the dense 16-bit MFMA peak.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0          # MI355X dense bf16/fp16 MFMA
MFMA_FP4_PEAK_TFLOPS = 10100.0     # MI355X dense FP4 MFMA (the MX variant's products)
MFMA_FP8_PEAK_TFLOPS = 5000.0      # MI355X dense FP8 MFMA (P V of the mixed recipe)
KERNEL_GEMMS = {"fwd_train": 6.0, "fwd_infer": 4.0, "fwd_infer_mx": 4.0, "fwd_infer_mx_fp8pv": 4.0, "bwd_dq": 6.0, "bwd_dkdv": 8.0}   # bwd_dkdv: see main()
# Sec. 3.4: peak forward throughput on B200 (NVFP4 QK + FP8 PV) at b=1, s=32768, h=32, d=128.  Another machine and
# another recipe: context for the forward on that shape, not a target.
PAPER_FWD_TFLOPS = {"paper_peak_fwd_shape": 2026.0}
# Bytes beyond L2 per launch of a kernel (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, factors from a 1 GiB copy kernel).  NOT measured
# by the run that prints them: they come from separate rocprofv3 --pmc runs of this same command, whose summaries (with
# the commit they were taken at) are the files named here; a kernel that changed since then has no entry.
def _traffic(gb, source):
    return {"bytes": gb * 1e9, "source": source}


TRAFFIC_BEYOND_L2 = {
    "dit720p_train": {k: _traffic(v, "profiles/hbm_traffic_dit720p_train.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, separate runs, scaled by "
                                     "the copy-kernel calibration; stored from that run, not collected live)")
                      for k, v in {"fwd_train": 17.5 + 4.51, "bwd_dq": 19.7 + 0.77, "bwd_dkdv": 310.8 + 1.55}.items()},
    "dit480p_infer": {"fwd_infer_mx": _traffic(0.883, "profiles/dit480p_infer_mx_fwd_kernels.txt (FETCH_SIZE, scaled; stored from that run)")},
}


HBM_PEAK_GBS = 8000.0              # MI355X HBM3E


def hbm_kernel_report(kern_ms, w, train):
    """Achieved GB/s of the bandwidth-bound kernels against the HBM peak.  Algorithmic bytes per element (d innermost):
    a quantization pass reads 2 B (bf16) and writes 2 B (the fp16/bf16 workspace copy the attention kernels read);
    delta reads dO (2 B) and O' (4 B) and, per row, L (4 B), and writes the {L, D} pair (8 B); bounds reads the V^F and dO
    copies (2 B each) and the pairs."""
    nq = float(w.B) * w.Hq * w.L * w.d
    nkv = float(w.B) * w.Hkv * w.L * w.d
    rows = float(w.B) * w.Hq * w.L
    byts = {"prep_qkv": 4.0 * (nq + 2 * nkv), "prep_qkvdo": 4.0 * (2 * nq + 2 * nkv),
            "delta": 6.0 * nq + 12.0 * rows, "bounds": 2.0 * (nq + nkv) + 8.0 * rows, "quantize": None}
    out = {}
    for name, b in byts.items():
        if name in kern_ms and b:
            gbs = b / (kern_ms[name] * 1e-3) / 1e9
            out[name] = {"ms": round(kern_ms[name], 4), "algorithmic_bytes": int(b), "GB/s": round(gbs, 1),
                         "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    return out


def measure(aq, torch, np, W, w, steps, warmup, fmt="nvfp4", opts=0, ablation=0, passes="auto", keep_inputs=False):
    """Time `steps` passes of the whole path on workload w (inputs resident in HBM) and the kernels of one pass."""
    fp8pv = fmt == "mx_fp8pv"
    mx = fmt == "mx" or fp8pv
    train = w.passes == "fwd+bwd" and passes == "auto" and not fp8pv and not (opts & 4)
    t0 = time.time()
    x = W.make_inputs(w, with_do=train)
    gen_s = time.time() - t0
    dev = lambda b: torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16)
    q, k, v = dev(x["q"]), dev(x["k"]), dev(x["v"])
    do = dev(x["do"]) if train else None
    B, Hq, Hkv, L, d = w.B, w.Hq, w.Hkv, w.L, w.d

    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, L), dtype=torch.float32, device="cuda")
    ohp = None
    if train:
        ohp = torch.empty((B, Hq, L, d), dtype=torch.float32, device="cuda")
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws_bytes = max(aq.workspace_bytes(aq.WS_FWD_MX if mx else aq.WS_FWD, B, Hq, Hkv, L, d),
                       aq.workspace_bytes(aq.WS_BWD_MX if mx else aq.WS_BWD, B, Hq, Hkv, L, d))
    else:
        ws_bytes = aq.workspace_bytes(aq.WS_FWD_INFER_MX_FP8PV if fp8pv else aq.WS_FWD_INFER_MX if mx else aq.WS_FWD,
                                      B, Hq, Hkv, L, d)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def fwd():
        if opts:
            aq.attnqat_fwd_opt(q, k, v, w.causal, opts, train=train, workspace=ws, out=(o, lse, ohp if train else None))
        elif train:
            (aq.attnqat_fwd_mx if mx else aq.attnqat_fwd)(q, k, v, w.causal, workspace=ws, out=(o, lse, ohp))
        elif fp8pv:
            aq.attnqat_fwd_infer_mx_fp8pv(q, k, v, w.causal, workspace=ws, out=(o, lse))
        elif mx:
            aq.attnqat_fwd_infer_mx(q, k, v, w.causal, workspace=ws, out=(o, lse))
        else:
            aq.attnqat_fwd_infer(q, k, v, w.causal, workspace=ws, out=(o, lse))

    def bwd():
        if opts:
            aq.attnqat_bwd_opt(q, k, v, do, lse, ohp, w.causal, opts, workspace=ws, out=(dq, dk, dv))
        elif ablation:
            aq.attnqat_bwd_ablation(q, k, v, do, lse, ohp, o, w.causal, ablation, workspace=ws, out=(dq, dk, dv))
        else:
            (aq.attnqat_bwd_mx if mx else aq.attnqat_bwd)(q, k, v, do, lse, ohp, w.causal, workspace=ws, out=(dq, dk, dv))

    def step():
        fwd()
        if train:
            bwd()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3

    # per-kernel durations: HIP events recorded by the library on the launch stream
    aq.profile_enable(True)
    kern_ms = {}
    nprof = max(1, min(steps, 3))
    for _ in range(nprof):
        fwd(); torch.cuda.synchronize()
        for name, ms in aq.profile_read():
            kern_ms[name] = kern_ms.get(name, 0.0) + ms / nprof
        if train:
            bwd(); torch.cuda.synchronize()
            for name, ms in aq.profile_read():
                kern_ms[name] = kern_ms.get(name, 0.0) + ms / nprof
    packed = None
    if fmt == "nvfp4" and not train and not opts:
        # Alg. 1 on already quantized inputs (the paper's inference numbers count the Q/K/V preprocessing, and that
        # preprocessing is where its speedup over SageAttention3 comes from: Sec. 3.4): the same forward with the
        # quantization pass replaced by the unpacking of the codes attnqat_quantize wrote
        packs = [aq.attnqat_quantize(t, want_xf=False)[:2] for t in (q, k, v)]
        torch.cuda.synchronize()
        aq.profile_enable(False)
        for _ in range(warmup):
            aq.attnqat_fwd_infer_packed(*packs, w.causal, d, workspace=ws, out=(o, lse))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            aq.attnqat_fwd_infer_packed(*packs, w.causal, d, workspace=ws, out=(o, lse))
        torch.cuda.synchronize()
        pms = (time.perf_counter() - t0) / steps * 1e3
        aq.profile_enable(True)
        aq.attnqat_fwd_infer_packed(*packs, w.causal, d, workspace=ws, out=(o, lse)); torch.cuda.synchronize()
        pk = dict(aq.profile_read())
        packed = {"ms_per_step": round(pms, 3), "tflops": round(w.fwd_flops / (pms * 1e-3) / 1e12, 2),
                  "unpack_qkv_ms": round(pk.get("unpack_qkv", 0.0), 4), "fwd_infer_ms": round(pk.get("fwd_infer", 0.0), 3)}
        del packs
    if fmt == "nvfp4":
        # the public quantizer on Q alone: 2 B read, 0.5 B of codes and 1/16 B of scale written per element
        codes = torch.empty((B, Hq, L, d // 2), dtype=torch.uint8, device="cuda")
        scales = torch.empty((B, Hq, L, d // 16), dtype=torch.uint8, device="cuda")
        qms = 0.0
        for _ in range(nprof + 1):
            aq.lib().attnqat_quantize(q.data_ptr(), B, Hq, L, d, aq.BF16, codes.data_ptr(), scales.data_ptr(), None,
                                      torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            qms = dict(aq.profile_read())["quantize"]          # the last (warm) call
        del codes, scales
    aq.profile_enable(False)
    pf_frac = None
    if train and (ablation & 2 or mx or opts & 2):
        pf_frac = 1.0                    # the un-quantized P is never skipped; an MX P^F tile is zero only if P itself is
    elif train:
        # how many 32x32 tiles of the dK/dV pass had a non-zero P^F (the others skip the dV products, exactly)
        counts = torch.zeros(2, dtype=torch.int64, device="cuda")
        aq.debug_dkdv_tile_counts(counts)
        bwd(); torch.cuda.synchronize()
        aq.debug_dkdv_tile_counts(None)
        visited, nonzero = (int(c) for c in counts.cpu())
        pf_frac = nonzero / max(visited, 1)

    pair_flops = B * Hq * float(L) ** 2 * d * (0.5 if w.causal else 1.0)
    step_flops = w.fwd_flops + (w.bwd_flops if train else 0.0)
    value = step_flops / (ms_per_step * 1e-3) / 1e12
    fwd_ms = sum(kern_ms.get(n, 0.0) for n in ("prep_qkv", "fwd_train", "fwd_infer", "prep_qkv_mx", "fwd_infer_mx", "fwd_infer_mx_fp8pv"))
    peak = MFMA_FP4_PEAK_TFLOPS if (mx and not train) else MFMA_PEAK_TFLOPS
    if fp8pv:      # half of the products at the FP4 rate, half at the FP8 rate
        peak = round(2.0 / (1.0 / MFMA_FP4_PEAK_TFLOPS + 1.0 / MFMA_FP8_PEAK_TFLOPS), 1)
    gemms = dict(KERNEL_GEMMS)
    if pf_frac is not None:
        gemms["bwd_dkdv"] = 6.0 + 2.0 * pf_frac
    dom = max((n for n in kern_ms if n in gemms), key=lambda n: kern_ms[n])
    achieved = gemms[dom] * pair_flops / (kern_ms[dom] * 1e-3) / 1e12
    traffic = TRAFFIC_BEYOND_L2.get(w.name, {}).get(dom) if (fmt == "nvfp4" and not opts and not ablation) or dom == "fwd_infer_mx" else None
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": peak,
                "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "traffic": traffic["bytes"] if traffic else None,
                "traffic_source": traffic["source"] if traffic else None,
                "kernel_ms": round(kern_ms[dom], 3),
                "dkdv_tiles_with_nonzero_pf": None if pf_frac is None else round(pf_frac, 6),
                "per_kernel": {n: {"ms": round(ms, 3),
                                   "tflops": round(gemms[n] * pair_flops / (ms * 1e-3) / 1e12, 2)
                                   if n in gemms else None} for n, ms in kern_ms.items()},
                "hbm_bound_kernels": hbm_kernel_report(kern_ms, w, train)}
    if fmt == "nvfp4":
        qb = float(B) * Hq * L * d * (2.0 + 0.5 + 0.0625)
        roofline["hbm_bound_kernels"]["quantize"] = {
            "ms": round(qms, 4), "algorithmic_bytes": int(qb), "GB/s": round(qb / (qms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(qb / (qms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "what": "attnqat_quantize on Q: codes and scales out, no dequantized copy"}
    fk = next((n for n in ("fwd_train", "fwd_infer", "fwd_infer_mx", "fwd_infer_mx_fp8pv") if n in kern_ms), None)
    roofline["forward"] = {"with_quantization_pass": {"ms": round(fwd_ms, 3), "tflops": round(w.fwd_flops / (fwd_ms * 1e-3) / 1e12, 2)},
                           "kernel_alone": {"ms": round(kern_ms[fk], 3), "tflops": round(w.fwd_flops / (kern_ms[fk] * 1e-3) / 1e12, 2)},
                           "from_packed_inputs": packed}
    res = {"train": train, "mx": mx, "fp8pv": fp8pv, "ms_per_step": ms_per_step, "value": value, "fwd_ms": fwd_ms, "peak": peak,
           "achieved": achieved, "gen_s": gen_s, "roofline": roofline, "x": x if keep_inputs else None}
    return res


def per_config_entry(w, r):
    """The short record of one benchmark configuration for the per_config array."""
    rf = r["roofline"]
    return {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "L": w.L, "d": w.d, "causal": w.causal,
            "passes": w.passes if r["train"] else "fwd_infer", "ms_per_step": round(r["ms_per_step"], 3),
            "fwd_tflops": round(w.fwd_flops / (r["fwd_ms"] * 1e-3) / 1e12, 2) if r["fwd_ms"] > 0 else None,
            "fwd_bwd_tflops": round(r["value"], 2) if r["train"] else None,
            "frac_of_mfma_peak_model_flops": round(r["value"] / r["peak"], 4),
            "dominant_kernel": {"kernel": rf["kernel"], "ms": rf["kernel_ms"], "executed_tflops": rf["achieved"], "frac": rf["frac"]},
            "dkdv_tiles_with_nonzero_pf": rf["dkdv_tiles_with_nonzero_pf"],
            "forward": rf["forward"],
            "kernel_ms": {n: v["ms"] for n, v in rf["per_kernel"].items()},
            "hbm_bound_kernels": {n: {"GB/s": v["GB/s"], "frac_of_hbm_peak": v["frac_of_hbm_peak"]} for n, v in rf["hbm_bound_kernels"].items()}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="dit720p_train",
                    help="one of: tiny_ref dit480p_infer llm4k_gqa dit720p_train llm32k_gqa; or paper_peak_fwd_shape "
                         "(context only: the shape of the paper's peak forward figure)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample (0 = skip)")
    ap.add_argument("--ablation", type=int, default=0,
                    help="backward ablation bit set of Sec. 3.2 (1: D from the bf16 O, 2: dV from the un-quantized P); "
                         "0 = the method itself")
    ap.add_argument("--format", default="nvfp4", choices=["nvfp4", "mx", "mx_fp8pv"],
                    help="nvfp4: the paper's format (default).  mx: E2M1 blocks of 32 with E8M0 scales: the inference "
                         "forward runs on the scaled FP4 MFMA, the training forward and the backward on the 16-bit path.  "
                         "mx_fp8pv: the mixed recipe (FP4 Q K^T, MXFP8 P V), inference forward only")
    ap.add_argument("--smooth-k", action="store_true",
                    help="K smoothing option of Sec. 3.2 (nvfp4 format only): phi on K minus its token mean")
    ap.add_argument("--two-level-p", action="store_true",
                    help="two-level quantization of P, the other option of Sec. 3.2 (nvfp4 format only)")
    ap.add_argument("--bf16-pv", action="store_true",
                    help="the mixed recipe of Sec. 2.5 (nvfp4 format only): NVFP4 Q K^T, P-tilde and V in bf16; inference forward only")
    ap.add_argument("--paged-lq", type=int, default=0,
                    help="serving mode (not a benchmark configuration): the forward over a paged FP4 KV cache (--format nvfp4 or mx) with this many "
                         "query positions per sequence (1 = a decode step) for 32 sequences of 4k-16k keys, 32 query / 8 kv heads")
    ap.add_argument("--sparse-keep", type=float, default=0.0,
                    help="block-sparse mode (not a benchmark configuration): the MX inference forward of the workload's shape "
                         "under a seeded random mask of 128 x 128 blocks that keeps this fraction (plus every query block's own block)")
    ap.add_argument("--mfma-sustained", action="store_true",
                    help="measurement only: the 16-bit MFMA rate and clock the part sustains with nothing else running "
                         "(context for the roofline fractions, which are quoted against the published 2.5 PFLOP/s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="measurement only: three launches of a plain 1 GiB copy kernel (reads 1 GiB, writes 1 GiB), the known-size "
                         "kernel against which rocprofv3's FETCH_SIZE / WRITE_SIZE are scaled")
    ap.add_argument("--passes", default="auto", choices=["auto", "fwd_infer"],
                    help="auto: the passes of the workload; fwd_infer: the inference forward (Alg. 1) on the workload's shape")
    ap.add_argument("--per-config", default="auto", choices=["auto", "on", "off"],
                    help="also time the other four benchmark configurations for a few steps each and report them in per_config "
                         "(auto: only in the default run, i.e. the headline workload in the paper's format without options)")
    args = ap.parse_args()
    if (args.smooth_k or args.two_level_p or args.bf16_pv) and (args.format != "nvfp4" or args.ablation):
        print("bench.py: --smooth-k, --two-level-p and --bf16-pv go with --format nvfp4 and no ablation", file=sys.stderr)
        sys.exit(2)
    if args.bf16_pv and args.two_level_p:
        print("bench.py: --bf16-pv leaves P-tilde un-blocked; it does not go with --two-level-p", file=sys.stderr)
        sys.exit(2)
    opts = (1 if args.smooth_k else 0) | (2 if args.two_level_p else 0) | (4 if args.bf16_pv else 0)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(heads shard across GPUs without communication, see DESIGN.md)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2603_00040_amd as aq
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    if args.mfma_sustained:
        from paper_2603_00040_amd import benchaux
        tf, ghz = benchaux.mfma_sustained()
        print(json.dumps({"metric": "sustained v_mfma_f32_32x32x16_f16 rate, register operands, 2 waves per SIMD (1 MI355X)",
                          "value": round(tf, 1), "unit": "TFLOP/s", "n_gpus": 1, "clock_ghz": round(ghz, 3),
                          "published_peak": MFMA_PEAK_TFLOPS, "frac_of_published_peak": round(tf / MFMA_PEAK_TFLOPS, 4)}), flush=True)
        return
    if args.copy_calibration:
        from paper_2603_00040_amd import benchaux
        nbytes, ms = benchaux.copy_calibration()
        print(json.dumps({"metric": "plain copy kernel (1 MI355X)", "value": round(2.0 * nbytes / (ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                          "n_gpus": 1, "bytes_read_per_launch": nbytes, "bytes_written_per_launch": nbytes, "launches": 3,
                          "kernel": "copy16_kernel", "ms": round(ms, 4)}), flush=True)
        return
    if args.paged_lq > 0:
        return bench_paged(args, aq, torch, np)
    w = W.by_name(args.workload)
    if args.sparse_keep > 0:
        return bench_sparse(args, aq, torch, np, w, W)

    r = measure(aq, torch, np, W, w, args.steps, args.warmup, args.format, opts, args.ablation, args.passes, keep_inputs=True)
    train, mx, fp8pv, value, peak, roofline = r["train"], r["mx"], r["fp8pv"], r["value"], r["peak"], r["roofline"]

    # what this machine sustains on MFMAs alone (boxes of one pool differ by 10 % in the clock they hold under load)
    try:
        from paper_2603_00040_amd import benchaux
        sus_tf, sus_ghz = benchaux.mfma_sustained(rounds=2, iters=20000)
        if peak == MFMA_PEAK_TFLOPS:
            roofline["mfma_sustained_on_this_box"] = {"tflops": round(sus_tf, 1), "clock_ghz": round(sus_ghz, 3),
                                                      "achieved_over_sustained": round(r["achieved"] / sus_tf, 4)}
    except Exception as e:       # context only: never fails the run
        roofline["mfma_sustained_on_this_box"] = {"error": str(e)}

    cpu = None
    if args.cpu_seconds > 0:
        cpu = cpu_baseline(w, r["x"], train, args.cpu_seconds, aq.block_k(), mx, fp8pv, args.smooth_k, args.two_level_p, args.bf16_pv)
    r["x"] = None

    # the other benchmark configurations, a few steps each (the headline line above stays the one `value` refers to)
    per_config = None
    default_run = w.name == "dit720p_train" and args.format == "nvfp4" and not opts and not args.ablation and args.passes == "auto"
    if args.per_config == "on" or (args.per_config == "auto" and default_run):
        per_config = []
        for wc in W.CONFIGS:
            if wc.name == w.name:
                per_config.append(per_config_entry(w, r))
                continue
            torch.cuda.empty_cache()
            rc = measure(aq, torch, np, W, wc, 5 if wc.L <= 40000 else 2, 2 if wc.L <= 40000 else 1, args.format, opts, args.ablation, "auto")
            per_config.append(per_config_entry(wc, rc))

    B, Hq, Hkv, L, d = w.B, w.Hq, w.Hkv, w.L, w.d
    out = {
        "metric": "FP4-attention fwd+bwd TFLOPS (1 MI355X)" if train else "FP4-attention fwd TFLOPS (1 MI355X)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(r["ms_per_step"], 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": round(value / PAPER_FWD_TFLOPS[w.name], 4) if (w.name in PAPER_FWD_TFLOPS and not train) else None,
        "dtype": "fp4 Q K^T, fp8 (E4M3) P V MFMA operands with E8M0 block scales, fp32 accumulate and softmax" if fp8pv
                 else "f16 MFMA on exact NVFP4 values for Q K^T, bf16 MFMA for P V, fp32 accumulate and softmax" if args.bf16_pv
                 else "fp4 (E2M1 codes with E8M0 block scales) MFMA operands, fp32 accumulate and softmax" if (mx and not train)
                 else "f16/bf16 MFMA operands (exact %s values), fp32 accumulate and softmax" % ("MXFP4" if mx else "NVFP4"),
        "data": "synthetic",
        "config": {"workload": w.name, "B": B, "Hq": Hq, "Hkv": Hkv, "L": L, "d": d, "causal": w.causal,
                   "passes": w.passes if train else "fwd_infer", "block_k": aq.block_k(), "seed": w.seed,
                   "bwd_ablation": args.ablation, "format": args.format, "smooth_k": bool(args.smooth_k), "two_level_p": bool(args.two_level_p),
                   "bf16_pv": bool(args.bf16_pv)},
        "fwd_tflops": round(w.fwd_flops / (r["fwd_ms"] * 1e-3) / 1e12, 2) if r["fwd_ms"] > 0 else None,
        "fwd_ms": round(r["fwd_ms"], 3),
        "frac_of_mfma_peak_model_flops": round(value / peak, 4),
        "input_gen_s": round(r["gen_s"], 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "per_config": per_config,
    }
    print(json.dumps(out), flush=True)


def bench_paged(args, aq, torch, np):
    """Serving shapes: 32 sequences with 4096..16384 keys (seeded), Hq = 32, Hkv = 8, d = 128, causal; the KV cache is
    written once (untimed), a step is one attnqat_fwd_infer_paged (--format nvfp4) or attnqat_fwd_infer_mx_paged (--format mx)
    call over all sequences."""
    B, Hq, Hkv, d, Lq = 32, 32, 8, 128, args.paged_lq
    nv = args.format == "nvfp4"
    page_bytes = (aq.kv_cache_page_bytes_nvfp4 if nv else aq.kv_cache_page_bytes)(Hkv, d)
    rng = np.random.default_rng(7)
    kv_lens = rng.integers(4096, 16385, B).astype(np.int32)
    kv_lens = np.maximum(kv_lens, Lq)
    max_pages = int((kv_lens.max() + 127) // 128)
    pages_of = [(int(n) + 127) // 128 for n in kv_lens]
    num_pages = sum(pages_of)
    perm = rng.permutation(num_pages).astype(np.int32)
    table = np.zeros((B, max_pages), np.int32)
    cache = torch.empty(num_pages * page_bytes, dtype=torch.uint8, device="cuda")
    import workloads as W
    dev = lambda bits: torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    nxt = 0
    qb = []
    for b in range(B):          # inputs from the seeded host generator, as everywhere else: N(0,1), K with 4 outlier channels x20
        n = int(kv_lens[b])
        table[b, :pages_of[b]] = perm[nxt:nxt + pages_of[b]]; nxt += pages_of[b]
        k = dev(W.fill(1, Hkv, n, d, 500 + b, W.TENSOR_K, "normal", 1.0, n_chan=4, chan_mult=20.0))
        v = dev(W.fill(1, Hkv, n, d, 500 + b, W.TENSOR_V, "normal", 1.0))
        qb.append(W.fill(1, Hq, Lq, d, 500 + b, W.TENSOR_Q, "normal", 1.0)[0])
        ids = torch.from_numpy(table[b, :pages_of[b]].copy()).cuda()
        if nv:
            aq.attnqat_kv_cache_write(k, v, cache, ids, 0, num_pages)
        else:
            aq.attnqat_kv_cache_write_mx(k, v, cache, ids, num_pages)
    q = dev(np.ascontiguousarray(np.stack(qb)))
    tab, lens = torch.from_numpy(table).cuda(), torch.from_numpy(kv_lens).cuda()
    o = torch.empty_like(q); lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device="cuda")
    if nv:
        ws = torch.empty(aq.lib().attnqat_paged_workspace_bytes(B, Hq, Hkv, Lq, max_pages, d), dtype=torch.uint8, device="cuda")
        step = lambda: aq.attnqat_fwd_infer_paged(q, cache, num_pages, tab, lens, Hkv, True, workspace=ws, out=(o, lse))
    else:
        ws = torch.empty(aq.workspace_bytes(aq.WS_FWD_INFER_MX_PAGED, B, Hq, Hkv, Lq, d), dtype=torch.uint8, device="cuda")
        step = lambda: aq.attnqat_fwd_infer_mx_paged(q, cache, num_pages, tab, lens, Hkv, True, workspace=ws, out=(o, lse))
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    aq.profile_enable(True)
    step(); torch.cuda.synchronize()
    kern = dict(aq.profile_read())
    aq.profile_enable(False)
    kname = next(n for n in ("decode_paged", "fwd_infer_paged", "fwd_infer_mx_paged") if n in kern)
    kms = kern[kname]
    # causal chunk: query i of the last Lq positions sees kv_len - Lq + i + 1 keys
    pairs = float(sum(Hq * (Lq * (int(n) - Lq) + Lq * (Lq + 1) / 2) for n in kv_lens))
    flops = 4.0 * pairs * d
    cache_bytes = float(sum(pages_of)) * page_bytes          # every page of every sequence, once
    decode = Lq <= 16 if not nv else kname == "decode_paged"
    mfma_peak = MFMA_PEAK_TFLOPS if nv else MFMA_FP4_PEAK_TFLOPS
    roofline = ({"bound": "hbm", "kernel": kname, "achieved": round(cache_bytes / (kms * 1e-3) / 1e9, 1), "peak": 8000.0,
                 "unit": "GB/s", "frac": round(cache_bytes / (kms * 1e-3) / 8e12, 4), "traffic": None, "kernel_ms": round(kms, 3)}
                if decode else
                {"bound": "mfma", "kernel": kname, "achieved": round(flops / (kms * 1e-3) / 1e12, 2), "peak": mfma_peak,
                 "unit": "TFLOP/s", "frac": round(flops / (kms * 1e-3) / 1e12 / mfma_peak, 4), "traffic": None, "kernel_ms": round(kms, 3)})
    print(json.dumps({
        "metric": "FP4-attention fwd TFLOPS (1 MI355X)", "value": round(flops / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 MFMA operands (exact NVFP4 values), fp32 accumulate and softmax" if nv
                 else "fp4 (E2M1 codes with E8M0 block scales) MFMA operands, fp32 accumulate and softmax", "data": "synthetic",
        "config": {"workload": "serving_paged_kv (not a benchmark configuration)", "B": B, "Hq": Hq, "Hkv": Hkv, "d": d, "Lq": Lq,
                   "kv_len_min": int(kv_lens.min()), "kv_len_max": int(kv_lens.max()), "kv_len_sum": int(kv_lens.sum()), "causal": True,
                   "page_keys": 128, "cache_bytes": int(cache_bytes), "format": args.format},
        "tokens_per_s": round(B * Lq / (ms * 1e-3), 1), "per_kernel_ms": {k_: round(v_, 3) for k_, v_ in kern.items()},
        "roofline": roofline, "cpu_baseline": None}), flush=True)


def bench_sparse(args, aq, torch, np, w, W):
    """Block-sparse MX forward on the workload's shape: a seeded random mask of 128 x 128 blocks; the flops counted are
    those of the blocks kept (below the diagonal only, if causal)."""
    B, Hq, Hkv, L, d = w.B, w.Hq, w.Hkv, w.L, w.d
    x = W.make_inputs(w, with_do=False)
    dev = lambda b: torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16)
    q, k, v = dev(x["q"]), dev(x["k"]), dev(x["v"])
    nb = (L + 127) // 128
    rng = np.random.default_rng(w.seed)
    bm = (rng.random((B, Hq, nb, nb)) < args.sparse_keep).astype(np.uint8)
    bm[:, :, np.arange(nb), np.arange(nb)] = 1
    if w.causal:
        bm *= np.tril(np.ones((nb, nb), np.uint8))
    edge = np.minimum(128, L - 128 * np.arange(nb)).astype(np.float64)              # rows / keys of every block
    pairs = edge[:, None] * edge[None, :]
    if w.causal:
        pairs[np.arange(nb), np.arange(nb)] = edge * (edge + 1) / 2
    kept_pairs = float((bm.astype(np.float64) * pairs).sum())
    mask = torch.from_numpy(bm).cuda()
    o = torch.empty_like(q); lse = torch.empty((B, Hq, L), dtype=torch.float32, device="cuda")
    ws = torch.empty(aq.workspace_bytes(aq.WS_FWD_INFER_MX_SPARSE, B, Hq, Hkv, L, d), dtype=torch.uint8, device="cuda")
    step = lambda: aq.attnqat_fwd_infer_mx_sparse(q, k, v, w.causal, mask, workspace=ws, out=(o, lse))
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    aq.profile_enable(True)
    step(); torch.cuda.synchronize()
    kern = dict(aq.profile_read())
    aq.profile_enable(False)
    kms = kern["fwd_infer_mx_sparse"]
    flops = 4.0 * kept_pairs * d
    print(json.dumps({
        "metric": "FP4-attention fwd TFLOPS (1 MI355X)", "value": round(flops / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp4 (E2M1 codes with E8M0 block scales) MFMA operands, fp32 accumulate and softmax", "data": "synthetic",
        "config": {"workload": w.name + " under a random block mask (not a benchmark configuration)", "B": B, "Hq": Hq, "Hkv": Hkv, "L": L,
                   "d": d, "causal": w.causal, "mask_block": [128, 128], "blocks_kept": round(float(bm.mean()), 4), "format": "mx"},
        "per_kernel_ms": {k_: round(v_, 3) for k_, v_ in kern.items()},
        "roofline": {"bound": "mfma", "kernel": "fwd_infer_mx_sparse", "achieved": round(flops / (kms * 1e-3) / 1e12, 2),
                     "peak": MFMA_FP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(flops / (kms * 1e-3) / 1e12 / MFMA_FP4_PEAK_TFLOPS, 4),
                     "traffic": None, "kernel_ms": round(kms, 3)},
        "cpu_baseline": None}), flush=True)


def cpu_baseline(w, x, train, target_s, block_k, mx=False, fp8pv=False, smooth_k=False, two_level=False, bf16pv=False):
    """Time the oracle (as it stands) on a bounded sample of the same workload: the forward of sampled query rows and,
    for training workloads, their dQ and their contributions to dK and dV over all keys (the whole of Alg. 3 for those
    rows: 14 model FLOPs per row-key-d with the forward)."""
    import numpy as np

    import oracle
    import workloads as W
    rng = np.random.default_rng(12345)
    # one head keeps the host copies small; rows are spread over the whole sequence
    b, h = 0, 0
    hk = h // (w.Hq // w.Hkv)
    f = {n: W.bf16_bits_to_f32(x[n][b:b + 1, (h if n in ("q", "do") else hk):(h if n in ("q", "do") else hk) + 1])
         for n in x}
    if smooth_k:
        f["k"] = oracle.smooth_k(f["k"])
    per_row = (4.0 + (10.0 if train else 0.0)) * w.L * w.d * (0.5 if w.causal else 1.0)

    def run(n):
        rows = np.sort(rng.choice(w.L, size=min(n, w.L), replace=False)).astype(np.int64)
        t0 = time.perf_counter()
        sm = oracle.MX_FP8PV if fp8pv else oracle.MX if mx else oracle.TWO_LEVEL_P if two_level else oracle.BF16_PV if bf16pv else 0
        r = oracle.fwd(f["q"], f["k"], f["v"], w.causal, block_k, scale_mode=sm, rows=rows)
        if train:
            oracle.bwd_dq_rows(f["q"], f["k"], f["v"], f["do"], rows, r["L"], r["Op"], w.causal, scale_mode=sm)
            oracle.bwd_rows_dkdv(f["q"], f["k"], f["v"], f["do"], rows, r["L"], r["Op"], w.causal, scale_mode=sm)
        return rows.size, time.perf_counter() - t0

    # two pilots separate the fixed cost (phi of the head's Q/K/V) from the cost per row
    n1, t1 = run(16)
    n2, t2 = run(min(w.L, 512))
    per = max((t2 - t1) / max(n2 - n1, 1), 1e-5)
    fixed = max(t1 - per * n1, 0.0)
    n = int(max(48, min(w.L, (target_s - fixed) / per)))
    n, t = run(n)
    return {"value": round(n * per_row / t / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{n} query rows of head (0,0), all {w.L} keys: oracle forward"
                      + (" + oracle dQ of those rows + their dK, dV contributions over all keys (model FLOPs 4+10 per row-key-d)"
                         if train else " (model FLOPs 4 per row-key-d)")
                      + f", {t:.1f} s, includes phi of that head's Q/K/V"}


if __name__ == "__main__":
    main()
