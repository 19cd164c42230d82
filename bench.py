#!/usr/bin/env python3
"""Benchmark of the attention hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input:
fa_fwd (Algorithm 1) followed by fa_bwd (Algorithm 2: D pre-pass, dK/dV kernel, dQ
kernel) on the workload named in `config.workload`, inputs resident in HBM.
Workloads with two lengths run fa_cross_fwd + fa_cross_bwd; workloads with a
handful of query rows against a long cache run fa_splitkv_fwd alone and report
GB/s of compulsory traffic against the HBM roofline. Throughput is
counted with the paper's formula (section 4.1): forward 4*N^2*d FLOPs per head
and sequence, halved under the causal mask, backward 2.5x that.

Prints ONE JSON line. Besides the contract fields it carries
  roofline     - the dominant kernel (backward dK/dV) against the bf16 MFMA peak: the
                 FLOPs of the four products it performs divided by its duration, which
                 is measured with HIP events inside the timed loop;
  roofline_fwd, roofline_dq - the same for the forward and the dQ kernels;
  mfma_loop    - TFLOP/s and shader clock of a register-resident loop of the same MFMA on
                 constant and on pseudo-random operands: what the pipe sustains on this machine;
  cpu_baseline - the float64 oracle timed on the host cores on a bounded sample;
  sweep        - (default workload only, after the timed region) the paper's benchmark grid
                 (section 4.1: 16k tokens, hidden 2048, d = 64 with 32 heads and d = 128 with 16,
                 N = 512 .. 16k, with and without the causal mask): forward and forward+backward
                 TFLOPs/s of every point, so that one run carries the whole metric. The headline
                 `value` stays the single workload named in `config`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak

# HBM bytes per launch (read + written) from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes recorded
# under profiles/pmc_<workload>_kernels.md, already scaled by the copy-kernel factors given there.
# A counter pass cannot run inside this script; workloads without a recorded pass report null.
MEASURED_TRAFFIC = {
    "d128_n8k_causal": {"fwd_kernel": 647689454, "bwd_dkdv_kernel": 828062947, "bwd_dq_kernel": 740116376},
    "sweep_d128_n8192_full": {"fwd_kernel": 269784965, "bwd_dkdv_kernel": 405079995, "bwd_dq_kernel": 337935017},
    "sweep_d64_n8192_causal": {"fwd_kernel": 884646395, "bwd_dkdv_kernel": 879984373, "bwd_dq_kernel": 830892697},
    "d256_n8k_causal": {"fwd_kernel": 791084128, "bwd_dkdv_kernel": 898424133, "bwd_dq_kernel": 772954746},  # fwd256 / dkdv256 / dq256
    "decode_b8_on_8k": {"fwd_kernel": 288777216},  # split kernel + merge, profiles/bench_decode_b8_on_8k_kernel_stats.md
}


def cpu_baseline(prob, budget_s: float = 12.0):
    """Time the float64 oracle (forward + backward) on as many (sequence, head)
    units of the workload as fit in about `budget_s` seconds, all host cores,
    and scale to the metric's unit with the same FLOP formula."""
    import numpy as np
    from oracle import attention_oracle as orc

    cores = len(os.sched_getaffinity(0))
    G = prob.Hq // prob.Hkv
    units = []
    t0 = time.perf_counter()
    for (b, h) in [(b, h) for b in range(prob.B) for h in range(prob.Hq)]:
        if units and time.perf_counter() - t0 > budget_s:
            break
        units.append((b, h))
        q = orc.widen_bf16(prob.Q[b, :, h])
        k = orc.widen_bf16(prob.K[b, :, h // G])
        v = orc.widen_bf16(prob.V[b, :, h // G])
        do = orc.widen_bf16(prob.dO[b, :, h])
        orc.head_backward(q, k, v, do, prob.scale, prob.causal)  # recomputes the forward inside
    dt = time.perf_counter() - t0
    per_unit = 3.5 * prob.fwd_flops() / (prob.B * prob.Hq)  # the metric's forward + backward FLOPs of one unit
    return {
        "value": per_unit * len(units) / dt / 1e12,
        "unit": "TFLOPs/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"{len(units)} of {prob.B * prob.Hq} (sequence, head) units of {prob.name}, forward+backward, "
                  f"float64 numpy, {dt:.1f} s",
    }


def paper_grid(binding, torch, samples: int = 20, warmup: int = 5):
    """Forward and forward+backward TFLOPs/s over the grid of section 4.1. Inputs are drawn on the
    GPU (N(0,1) rounded to bf16, seeded): the values do not change the work. Per point: `warmup`
    calls, then the median of `samples` timed batches (short calls are timed several at a time:
    a batch lasts about a millisecond)."""
    import statistics
    gen = torch.Generator(device="cuda").manual_seed(1002)
    out = {}
    for d, H in ((64, 32), (128, 16)):
        for N in (512, 1024, 2048, 4096, 8192, 16384):
            B = 16384 // N
            Q, K, V, dO = (torch.randn(B, N, H, d, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(4))
            O = torch.empty_like(Q)
            LSE = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
            dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
            ws = torch.empty(binding.fa_bwd_workspace_bytes(B, H, H, N, d), dtype=torch.uint8, device="cuda")
            sc = d ** -0.5
            for causal in (False, True):
                def fwd():
                    binding.fa_fwd(Q, K, V, sc, causal, O=O, LSE=LSE)

                def both():
                    fwd()
                    binding.fa_bwd(Q, K, V, O, dO, LSE, sc, causal, dQ=dQ, dK=dK, dV=dV, workspace=ws)

                ms = []
                for fn in (fwd, both):
                    def timed(k):
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        for _ in range(k):
                            fn()
                        e1.record()
                        torch.cuda.synchronize()
                        return e0.elapsed_time(e1) / k
                    for _ in range(warmup):
                        fn()
                    k = max(1, min(16, int(1.0 / max(timed(1), 1e-3))))
                    ms.append(statistics.median(timed(k) for _ in range(samples)))
                fl = 4.0 * B * H * N * N * d * (0.5 if causal else 1.0)
                out[f"d{d}_n{N}_{'causal' if causal else 'full'}"] = {
                    "fwd_tflops": round(fl / ms[0] / 1e9, 1), "fwd_bwd_tflops": round(3.5 * fl / ms[1] / 1e9, 1)}
    return out


def bench_decode(args, prob, binding) -> int:
    """Few query rows against a long key/value cache: one step is one fa_splitkv_fwd call (the split
    kernel and the merge). HBM-bound: the roofline is bytes that must move over the call's duration."""
    import numpy as np
    import torch

    def gpu(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    Q, K, V = (gpu(x) for x in (prob.Q, prob.K, prob.V))
    B, Nq, Hq, d = Q.shape
    splits = binding.splitkv_default_splits(B, Hq, prob.Hkv, Nq, prob.Nk)
    O = torch.empty_like(Q)
    LSE = torch.empty((B, Hq, Nq), dtype=torch.float32, device="cuda")
    ws = torch.empty(binding.fa_splitkv_fwd_workspace_bytes(B, Hq, Nq, d, splits), dtype=torch.uint8, device="cuda")

    def step():
        binding.fa_splitkv_fwd(Q, K, V, prob.scale, prob.causal, splits, O=O, LSE=LSE, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kern_ms = e0.elapsed_time(e1) / args.steps
    # bytes that must move: K and V once, Q read and O written once, LSE written
    alg_bytes = 2.0 * (K.numel() + V.numel() + Q.numel() + O.numel()) + 4.0 * LSE.numel()
    gbs = alg_bytes / (kern_ms * 1e-3) / 1e9
    out = {
        "metric": "decode attention forward, GB/s of compulsory traffic (bf16)", "value": alg_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": prob.name, "B": B, "Nq": Nq, "Nk": prob.Nk, "Hq": Hq, "Hkv": prob.Hkv, "d": d,
                   "causal": prob.causal, "num_splits": splits, "algorithmic_bytes": alg_bytes},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": 8000.0, "unit": "GB/s", "frac": gbs / 8000.0,
                     "traffic": MEASURED_TRAFFIC.get(prob.name, {}).get("fwd_kernel"), "avg_kernel_ms": kern_ms,
                     "kernel": "fwd_kernel<.., split> + fwd_merge_kernel"},
    }
    if not args.no_cpu_baseline:
        from oracle import attention_oracle as orc
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < 10.0:
            b = n % B
            orc.attention_forward(orc.widen_bf16(prob.Q[b:b + 1]), orc.widen_bf16(prob.K[b:b + 1]),
                                  orc.widen_bf16(prob.V[b:b + 1]), prob.scale, prob.causal)
            n += 1
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": alg_bytes / B * n / dt / 1e9, "unit": "GB/s", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": f"{n} sequence passes of {prob.name} (all heads), forward, float64 numpy, {dt:.1f} s"}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="d128_n8k_causal")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fwd-only", action="store_true", help="profiling aid: time the forward alone")
    ap.add_argument("--no-sweep", action="store_true", help="skip the grid of section 4.1 after the timed region")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="profiling aid: instead of the benchmark, run 5 device-to-device copies of BYTES bytes; "
                         "under rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE they give the counters' scale factors")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2307_08691_amd import binding, inputs

    binding.load()
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.full((args.copy_calibration,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": args.copy_calibration, "copies": 5}))
        return 0
    prob = inputs.make_config(args.workload)
    if prob.varlen:
        print("bench.py: pick a dense workload", file=sys.stderr)
        return 2
    if prob.Nk and prob.N * (prob.Hq // prob.Hkv) <= 256:
        return bench_decode(args, prob, binding)

    def gpu(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    Q, K, V, dO = (gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    B, N, Hq, d = Q.shape
    O = torch.empty_like(Q)
    LSE = torch.empty((B, Hq, N), dtype=torch.float32, device="cuda")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    ws = torch.empty(binding.fa_bwd_workspace_bytes(B, Hq, prob.Hkv, N, d), dtype=torch.uint8, device="cuda")
    sc, ca = prob.scale, prob.causal

    def step(ev=None):
        """fa_fwd + the three backward launches, in the order fa_bwd issues them; with `ev`
        the forward, dK/dV and dQ kernels are bracketed by events."""
        if ev:
            ev[0].record()
        if prob.Nk:  # two lengths: one call per pass, the backward is not taken apart
            binding.fa_cross_fwd(Q, K, V, sc, ca, O=O, LSE=LSE)
            if ev:
                ev[1].record()
            if not args.fwd_only:
                binding.fa_cross_bwd(Q, K, V, O, dO, LSE, sc, ca, dQ=dQ, dK=dK, dV=dV, workspace=ws)
            if ev:
                for e in ev[2:]:
                    e.record()
            return
        binding.fa_fwd(Q, K, V, sc, ca, O=O, LSE=LSE)
        if ev:
            ev[1].record()
        if args.fwd_only:
            return
        binding.fa_bwd_stages(Q, K, V, O, dO, LSE, sc, ca, 1, dQ, dK, dV, ws)
        if ev:
            ev[2].record()
        binding.fa_bwd_stages(Q, K, V, O, dO, LSE, sc, ca, 2, dQ, dK, dV, ws)
        if ev:
            ev[3].record()
        binding.fa_bwd_stages(Q, K, V, O, dO, LSE, sc, ca, 4, dQ, dK, dV, ws)
        if ev:
            ev[4].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # events are recorded on torch's current stream, the one the kernels are launched on
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    fwd_fl, bwd_fl = prob.fwd_flops(), prob.bwd_flops()
    total_fl = fwd_fl if args.fwd_only else fwd_fl + bwd_fl
    value = total_fl / (ms_per_step * 1e-3) / 1e12

    def roof(flops, ms, kernel):
        ach = flops / (ms * 1e-3) / 1e12
        return {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_BF16_TFLOPS, "traffic": MEASURED_TRAFFIC.get(prob.name, {}).get(kernel),
                "avg_kernel_ms": ms, "kernel": kernel}

    out = {
        "metric": "attention fwd+bwd TFLOPs/s (bf16)" if not args.fwd_only else "attention fwd TFLOPs/s (bf16)",
        "value": value,
        "unit": "TFLOPs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": prob.name, "B": B, "N": N, "Hq": Hq, "Hkv": prob.Hkv, "d": d, "causal": ca,
                   "scale": sc, "fwd_flops": fwd_fl, "bwd_flops": bwd_fl},
        "frac_of_bf16_peak": value / PEAK_BF16_TFLOPS,
        "roofline_fwd": roof(fwd_fl, fwd_ms, "fwd_kernel"),
    }
    if prob.Nk and not args.fwd_only:
        bwd_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps
        out["roofline"] = roof(3.5 * fwd_fl, bwd_ms, "bwd_prep_kernel + bwd_dkdv_kernel + bwd_dq_kernel")
        out["config"]["Nk"] = prob.Nk
    elif not args.fwd_only:
        # metric FLOPs count 5 products (2.5 x forward); the dK/dV kernel performs 4 of them
        # (S, dP, dV, dK) and the dQ kernel 3 (S, dP recomputed, dQ): 2 x and 1.5 x forward
        dkdv_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
        dq_ms = sum(e[3].elapsed_time(e[4]) for e in evs) / args.steps
        out["roofline"] = roof(2.0 * fwd_fl, dkdv_ms, "bwd_dkdv_kernel")
        out["roofline_dq"] = roof(1.5 * fwd_fl, dq_ms, "bwd_dq_kernel")
    else:
        out["roofline"] = out["roofline_fwd"]
    # what the matrix pipe sustains on this machine with every operand in registers (outside the timed region)
    out["mfma_loop"] = {}
    for key, rnd in (("constant_operands", False), ("random_operands", True)):
        tf, ghz = binding.fa_mfma_probe(2000, rnd)
        out["mfma_loop"][key] = {"tflops": tf, "shader_clock_ghz": ghz}
    if not args.no_sweep and not args.fwd_only and args.workload == "d128_n8k_causal":
        del Q, K, V, dO, O, LSE, dQ, dK, dV, ws
        out["sweep"] = paper_grid(binding, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(prob)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
