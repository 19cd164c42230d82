#!/usr/bin/env python3
"""Benchmark of the attention hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input, through the
entry points a user calls: the forward (Algorithm 1) followed by the backward (Algorithm 2: D
pre-pass, dK/dV kernel, dQ kernel) of the workload named in `config.workload`, inputs resident
in HBM. Dense workloads run fa_fwd + fa_bwd, packed ragged ones fa_varlen_fwd + fa_varlen_bwd,
workloads with two lengths fa_cross_*, half precision fa_cross_*_f16, dropout and mask workloads
their own entry points; a handful of query rows against a long cache runs fa_splitkv_fwd alone
and reports GB/s of compulsory traffic against the HBM roofline. Throughput is counted with the
paper's formula (section 4.1): forward 4*N^2*d FLOPs per head and sequence, halved under the
causal mask, backward 2.5x that.

Before the `--warmup` steps the same step runs untimed for `--settle` seconds (a fresh process on
an idle GPU otherwise measures the clock ramp). The timed region holds exactly `--steps` steps and
nothing else (no events inside). After it,
outside the timed region, the same number of forward calls and of backward calls are timed
apart with HIP events, and (dense bf16 workloads) every backward kernel on its own through
fa_bwd_stages: those per-kernel durations feed the roofline objects.

Prints ONE JSON line. Besides the contract fields it carries
  fwd, bwd     - TFLOPs/s, ms and fraction of the bf16 MFMA peak of the two passes timed apart;
  roofline     - the dominant kernel (backward dK/dV) against the bf16 MFMA peak: the FLOPs of
                 the four products it performs divided by its average duration;
  roofline_fwd, roofline_dq - the same for the forward and the dQ kernels;
  mfma_loop    - TFLOP/s and shader clock of a register-resident loop of the same MFMA on
                 constant and on pseudo-random operands: what the pipe sustains on this machine;
  cpu_baseline - the float64 oracle timed on the host cores on a bounded sample;
  configs      - (default workload only) forward / backward / both for the three single
                 workloads of the metric: d = 128 N = 8192 causal, the long x3 sequence, the
                 grouped-head ragged batch;
  sweep        - (default workload only) the paper's benchmark grid (section 4.1: 16k tokens,
                 hidden 2048, d = 64 with 32 heads and d = 128 with 16, N = 512 .. 16k, with and
                 without the causal mask): forward, backward and forward+backward TFLOPs/s and the
                 fractions of peak at every point, so that one run carries the whole metric. The
                 headline `value` stays the single workload named in `config`.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 / fp16 MFMA peak
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E peak

# HBM bytes per launch (read + written) from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes recorded
# under profiles/pmc_<workload>_kernels.md, already scaled by the copy-kernel factors given there.
# A counter pass cannot run inside this script, so the figures are only reported as `traffic` while
# the kernel sources are the ones they were measured on (`sources`: kernel_sources_id() at the time
# of the measurement); otherwise `traffic` is null and the stale figure moves to `traffic_recorded`.
MEASURED_TRAFFIC = {
    "sources": "aa63587ade56",
    "d128_n8k_causal": {"fwd_kernel": 657936517, "bwd_dkdv_kernel": 862384831, "bwd_dq_kernel": 736812614},
    "sweep_d128_n8192_full": {"fwd_kernel": 269806409, "bwd_dkdv_kernel": 405186020, "bwd_dq_kernel": 338038522},
    "sweep_d64_n8192_causal": {"fwd_kernel": 873743558, "bwd_dkdv_kernel": 883456292, "bwd_dq_kernel": 831791357},
    "decode_b8_on_8k": {"fwd_decode_kernel": 269316633},
    "decode_paged_b64_to_8k": {"fwd_decode_kernel": 1019765575},
}


def kernel_sources_id() -> str:
    """Short hash of the sources of the bf16 forward, backward and decode kernels (the ones the counter
    passes cover): identifies what a counter pass measured."""
    d = os.path.join(ROOT, "paper_2307_08691_amd", "csrc")
    h = hashlib.sha1()
    for f in ("fa_bwd.hip", "fa_common.h", "fa_decode.hip", "fa_fwd.hip", "fa_kernels.h", "fa_lds.h"):
        h.update(f.encode())
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:12]


def traffic_fields(workload: str, kernel: str) -> dict:
    rec = MEASURED_TRAFFIC.get(workload, {}).get(kernel)
    if rec is None:
        return {"traffic": None}
    if MEASURED_TRAFFIC["sources"] == kernel_sources_id():
        return {"traffic": rec, "traffic_from": f"profiles/{'bench' if workload.startswith('decode') else 'pmc'}_{workload}_{'kernel_stats' if workload.startswith('decode') else 'kernels'}.md"}
    return {"traffic": None, "traffic_recorded": {"bytes": rec, "profile": f"profiles/pmc_{workload}_kernels.md",
                                                  "kernel_sources": MEASURED_TRAFFIC["sources"],
                                                  "note": "measured on other kernel sources than this run's"}}


# ---------------------------------------------------------------------------------------------
# one workload on the GPU: its buffers and the calls of one step
# ---------------------------------------------------------------------------------------------

class Runner:
    """Buffers of one workload and the forward / backward calls of its entry points."""

    def __init__(self, prob, binding, torch, on_device=None):
        import numpy as np
        self.prob, self.b, self.torch = prob, binding, torch
        et = torch.float16 if prob.dtype == "f16" else torch.bfloat16

        def gpu(bits):
            return torch.from_numpy(bits.view(np.int16)).cuda().view(et)

        self.Q, self.K, self.V, self.dO = on_device if on_device is not None else (gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
        Q, K = self.Q, self.K
        self.O = torch.empty_like(Q)
        self.dQ, self.dK, self.dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(self.V)
        self.sc, self.ca = prob.scale, prob.causal
        self.stages = None
        self.drop = prob.meta.get("dropout")     # (p, seed) or None
        self.M = None
        if prob.varlen:
            T, Hq, d = Q.shape
            self.cu = torch.from_numpy(prob.cu_seqlens.astype(np.int32)).cuda()
            self.mx = int(prob.seqlens.max())
            self.LSE = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
            self.ws = torch.empty(binding.fa_varlen_bwd_workspace_bytes(T, Hq, prob.Hkv, d), dtype=torch.uint8, device="cuda")
            self.kind = "varlen_dropout" if self.drop else "varlen"
        else:
            B, N, Hq, d = Q.shape
            self.LSE = torch.empty((B, Hq, N), dtype=torch.float32, device="cuda")
            self.ws = torch.empty(binding.fa_cross_bwd_workspace_bytes(B, Hq, prob.Hkv, N, prob.keys, d), dtype=torch.uint8,
                                  device="cuda")
            if prob.meta.get("mask"):
                mk = prob.meta["mask"]
                gen = torch.Generator(device="cuda").manual_seed(mk["seed"])
                Hm = Hq if mk.get("per_head", True) else 1
                Bm = B if mk.get("per_sequence", True) else 1
                self.M = binding.mask_buffer(Bm, Hm, N, prob.keys)
                self.M.copy_(2.0 * torch.randn(Bm, Hm, N, prob.keys, device="cuda", generator=gen))
                gone = torch.rand(Bm, Hm, N, prob.keys, device="cuda", generator=gen) < mk.get("removed", 0.3)
                gone[..., 0] = False
                self.M.masked_fill_(gone, float("-inf"))
                del gone
                self.kind = "mask"
            elif self.drop:
                self.kind = "dropout"
            elif prob.meta.get("window"):
                self.kind = "local"
                self.win = prob.meta["window"]
            elif prob.meta.get("block_pattern"):
                from paper_2307_08691_amd import inputs
                bp = prob.meta["block_pattern"]
                self.kind = "blocksparse"
                self.block = bp["block"]
                self.BM = torch.from_numpy(inputs.block_pattern(bp["seed"], 1, Hq, N, prob.keys, bp["block"], bp["density"],
                                                                prob.causal).astype(np.uint8)).cuda()
            elif prob.Nk or prob.dtype == "f16":
                self.kind = "cross"
            else:
                self.kind = "dense"
                self.stages = lambda st: binding.fa_bwd_stages(self.Q, self.K, self.V, self.O, self.dO, self.LSE, self.sc,
                                                               self.ca, st, self.dQ, self.dK, self.dV, self.ws)

    def entry_points(self):
        return {"dense": "fa_fwd + fa_bwd", "cross": "fa_cross_fwd + fa_cross_bwd" + ("_f16" if self.prob.dtype == "f16" else ""),
                "varlen": "fa_varlen_fwd + fa_varlen_bwd", "dropout": "fa_dropout_fwd + fa_dropout_bwd",
                "varlen_dropout": "fa_varlen_dropout_fwd + fa_varlen_dropout_bwd", "mask": "fa_mask_fwd + fa_mask_bwd", "local": "fa_local_fwd + fa_local_bwd",
                "blocksparse": "fa_blocksparse_fwd + fa_blocksparse_bwd"}[self.kind]

    def fwd(self):
        b, k = self.b, self.kind
        a = (self.Q, self.K, self.V)
        if k == "dense":
            b.fa_fwd(*a, self.sc, self.ca, O=self.O, LSE=self.LSE)
        elif k == "cross":
            b.fa_cross_fwd(*a, self.sc, self.ca, O=self.O, LSE=self.LSE)
        elif k == "varlen":
            b.fa_varlen_fwd(*a, self.cu, self.mx, self.sc, self.ca, O=self.O, LSE=self.LSE)
        elif k == "dropout":
            b.fa_dropout_fwd(*a, self.sc, self.ca, *self.drop, O=self.O, LSE=self.LSE)
        elif k == "varlen_dropout":
            b.fa_varlen_dropout_fwd(*a, self.cu, self.mx, self.sc, self.ca, *self.drop, O=self.O, LSE=self.LSE)
        elif k == "local":
            b.fa_local_fwd(*a, self.sc, *self.win, O=self.O, LSE=self.LSE)
        elif k == "blocksparse":
            b.fa_blocksparse_fwd(*a, self.BM, self.block, self.sc, self.ca, O=self.O, LSE=self.LSE)
        else:
            b.fa_mask_fwd(*a, self.M, self.sc, self.ca, O=self.O, LSE=self.LSE)

    def bwd(self):
        b, k = self.b, self.kind
        a = (self.Q, self.K, self.V)
        out = dict(dQ=self.dQ, dK=self.dK, dV=self.dV, workspace=self.ws)
        if k == "dense":
            b.fa_bwd(*a, self.O, self.dO, self.LSE, self.sc, self.ca, **out)
        elif k == "cross":
            b.fa_cross_bwd(*a, self.O, self.dO, self.LSE, self.sc, self.ca, **out)
        elif k == "varlen":
            b.fa_varlen_bwd(*a, self.O, self.dO, self.LSE, self.cu, self.mx, self.sc, self.ca, **out)
        elif k == "dropout":
            b.fa_dropout_bwd(*a, self.O, self.dO, self.LSE, self.sc, self.ca, *self.drop, **out)
        elif k == "varlen_dropout":
            b.fa_varlen_dropout_bwd(*a, self.O, self.dO, self.LSE, self.cu, self.mx, self.sc, self.ca, *self.drop, **out)
        elif k == "local":
            b.fa_local_bwd(*a, self.O, self.dO, self.LSE, self.sc, *self.win, **out)
        elif k == "blocksparse":
            b.fa_blocksparse_bwd(*a, self.BM, self.block, self.O, self.dO, self.LSE, self.sc, self.ca, **out)
        else:
            b.fa_mask_bwd(*a, self.M, self.O, self.dO, self.LSE, self.sc, self.ca, **out)

    def both(self):
        self.fwd()
        self.bwd()

    def event_ms(self, fn, calls: int) -> float:
        """Average duration of `calls` back-to-back calls of fn, by HIP events on torch's current
        stream (the one the library launches on)."""
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(calls):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / calls


def three_rates(prob, fwd_ms, bwd_ms, both_ms):
    fl = prob.fwd_flops()
    r = {"fwd_ms": round(fwd_ms, 4), "bwd_ms": round(bwd_ms, 4), "fwd_bwd_ms": round(both_ms, 4),
         "fwd_tflops": round(fl / fwd_ms / 1e9, 1), "bwd_tflops": round(2.5 * fl / bwd_ms / 1e9, 1),
         "fwd_bwd_tflops": round(3.5 * fl / both_ms / 1e9, 1)}
    for k in ("fwd", "bwd", "fwd_bwd"):
        r[k + "_frac_of_peak"] = round(r[k + "_tflops"] / PEAK_BF16_TFLOPS, 4)
    if not prob.varlen:
        # What the HBM roofline (8 TB/s) allows for this shape: the credited FLOPs over the time the
        # bytes that the kernels must move would take (the per-kernel figures of the roofline object:
        # forward Q, O, K, V, L; dK/dV kernel Q, dO, L, D, K, V read and dK, dV written; dQ kernel Q, dO, O,
        # L, K, V read and dQ, D written). Below the MFMA peak for short sequences: those points are HBM-bound.
        B, N, Nk, Hq, Hkv, d = prob.B, prob.N, prob.keys, prob.Hq, prob.Hkv, prob.d
        by_f = B * Hq * (4 * N * d + 4 * N) + B * Hkv * 4 * Nk * d
        by_b = B * Hq * (4 * N * d + 8 * N) + B * Hkv * 8 * Nk * d + B * Hq * (8 * N * d + 12 * N) + B * Hkv * 4 * Nk * d
        for k, mult, by in (("fwd", 1.0, by_f), ("bwd", 2.5, by_b), ("fwd_bwd", 3.5, by_f + by_b)):
            r[k + "_hbm_bound_tflops"] = round(mult * fl / (by / (PEAK_HBM_GBS * 1e9)) / 1e12, 1)
    return r


def measure_config(name, binding, torch, inputs, calls=10, warmup=3):
    """Forward / backward / both of one named workload: `warmup` steps, then `calls` calls of each."""
    prob = inputs.make_config(name)
    r = Runner(prob, binding, torch)
    for _ in range(warmup):
        r.both()
    torch.cuda.synchronize()
    out = three_rates(prob, r.event_ms(r.fwd, calls), r.event_ms(r.bwd, calls), r.event_ms(r.both, calls))
    out["entry_points"] = r.entry_points()
    return out


def cpu_baseline(prob, budget_s: float = 12.0):
    """Time the float64 oracle (forward + backward) on as many (sequence, head)
    units of the workload as fit in about `budget_s` seconds, all host cores,
    and scale to the metric's unit with the same FLOP formula."""
    from oracle import attention_oracle as orc

    cores = len(os.sched_getaffinity(0))
    G = prob.Hq // prob.Hkv
    widen = orc.widen_f16 if prob.dtype == "f16" else orc.widen_bf16
    if prob.varlen:
        cu = prob.cu_seqlens
        todo = [(s, h) for s in range(len(cu) - 1) for h in range(prob.Hq)]
    else:
        todo = [(b, h) for b in range(prob.B) for h in range(prob.Hq)]
    done, pairs = 0, 0.0  # pairs: visible (query, key) pairs of the units done, as the metric counts them
    t0 = time.perf_counter()
    for (s, h) in todo:
        if done and time.perf_counter() - t0 > budget_s:
            break
        rows = slice(int(cu[s]), int(cu[s + 1])) if prob.varlen else (s, slice(None))
        q, k, v, do = (widen(x) for x in (prob.Q[rows][..., h, :], prob.K[rows][..., h // G, :], prob.V[rows][..., h // G, :],
                                          prob.dO[rows][..., h, :]))
        nq, nk = q.shape[0], k.shape[0]
        if nq == 0:
            continue
        orc.head_backward(q, k, v, do, prob.scale, prob.causal)  # recomputes the forward inside
        pairs += float(nq) * nk - (0.5 * float(nq) ** 2 if prob.causal else 0.0)
        done += 1
    flops = 3.5 * 4.0 * prob.d * pairs
    dt = time.perf_counter() - t0
    return {
        "value": flops / dt / 1e12,
        "unit": "TFLOPs/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"{done} of {len(todo)} (sequence, head) units of {prob.name}, forward+backward, "
                  f"float64 numpy, {dt:.1f} s",
    }


def paper_grid(binding, torch, inputs, samples: int = 20, warmup: int = 5):
    """Forward, backward and forward+backward TFLOPs/s over the grid of section 4.1. Inputs are drawn on
    the GPU (N(0,1) rounded to bf16, seeded): the values do not change the work. Per point: `warmup`
    calls, then the median of `samples` timed batches (short calls are timed several at a time:
    a batch lasts about a millisecond)."""
    gen = torch.Generator(device="cuda").manual_seed(1002)
    out = {}
    for d, H in ((64, 32), (128, 16)):
        for N in (512, 1024, 2048, 4096, 8192, 16384):
            B = 16384 // N
            dev = tuple(torch.randn(B, N, H, d, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(4))
            for causal in (False, True):
                prob = inputs.shape_only(B=B, N=N, Hq=H, Hkv=H, d=d, causal=causal, name=inputs.sweep_name(d, N, causal))
                r = Runner(prob, binding, torch, on_device=dev)
                ms = []
                for fn in (r.fwd, r.bwd, r.both):
                    for _ in range(warmup):
                        fn()
                    torch.cuda.synchronize()
                    k = max(1, min(16, int(1.0 / max(r.event_ms(fn, 1), 1e-3))))
                    ms.append(statistics.median(r.event_ms(fn, k) for _ in range(samples)))
                out[f"d{d}_n{N}_{'causal' if causal else 'full'}"] = three_rates(prob, *ms)
                del r
            del dev
    return out


def bench_fp8(args, prob, binding) -> int:
    """Forward on FP8 (E4M3) operands: one step is one fa_fp8_fwd call; roofline against the fp8 MFMA peak."""
    import torch
    dq, dk, dv = prob.meta["descale"]
    Q8, K8, V8 = (torch.from_numpy(x).cuda() for x in (prob.Q, prob.K, prob.V))
    Vt8 = binding.fp8_key_major(V8)
    B, Nq, Hq, d = Q8.shape
    O = torch.empty((B, Nq, Hq, d), dtype=torch.bfloat16, device="cuda")
    LSE = torch.empty((B, Hq, Nq), dtype=torch.float32, device="cuda")

    def step():
        binding.fa_fp8_fwd(Q8, K8, Vt8, prob.keys, prob.scale, dq, dk, dv, prob.causal, O=O, LSE=LSE)

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
    fl = prob.fwd_flops()
    ach = fl / kern_ms / 1e9
    out = {
        "metric": "attention fwd TFLOPs/s (fp8 e4m3 operands)", "value": fl / ms_per_step / 1e9, "unit": "TFLOPs/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp8", "data": "synthetic",
        "config": {"workload": prob.name, "B": B, "N": Nq, "Nk": prob.keys, "Hq": Hq, "Hkv": prob.Hkv, "d": d, "causal": prob.causal,
                   "fwd_flops": fl, "entry_points": "fa_fp8_fwd"},
        "roofline": {"bound": "mfma", "achieved": ach, "peak": 5000.0, "unit": "TFLOP/s", "frac": ach / 5000.0, "traffic": None,
                     "avg_kernel_ms": kern_ms, "kernel": "fwd_fp8_kernel"},
        "kernel_sources": kernel_sources_id(),
    }
    if not args.no_cpu_baseline:
        from oracle import attention_oracle as orc
        t0 = time.perf_counter()
        units = 0
        while time.perf_counter() - t0 < 10.0 and units < B * Hq:
            b, h = divmod(units, Hq)
            g = h // (Hq // prob.Hkv)
            orc.head_forward(dq * orc.widen_e4m3(prob.Q[b, :, h]), dk * orc.widen_e4m3(prob.K[b, :, g]),
                             dv * orc.widen_e4m3(prob.V[b, :, g]), prob.scale, prob.causal)
            units += 1
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": fl / (B * Hq) * units / dt / 1e12, "unit": "TFLOPs/s", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": f"{units} of {B * Hq} (sequence, head) units of {prob.name}, forward, float64 numpy, {dt:.1f} s"}
    print(json.dumps(out))
    return 0


def bench_decode(args, prob, binding) -> int:
    """Few query rows against a long key/value cache: one step is one fa_splitkv_fwd call (the split
    kernel and the merge). HBM-bound: the roofline is bytes that must move over the call's duration."""
    import numpy as np
    import torch

    def gpu(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    Q, K, V = (gpu(x) for x in (prob.Q, prob.K, prob.V))
    B, Nq, Hq, d = Q.shape
    splits = binding.splitkv_default_splits(B, Hq, prob.Hkv, Nq, prob.Nk, ragged=bool(prob.meta.get("cache")))
    O = torch.empty_like(Q)
    LSE = torch.empty((B, Hq, Nq), dtype=torch.float32, device="cuda")
    ws = torch.empty(binding.fa_splitkv_fwd_workspace_bytes(B, Hq, Nq, d, splits), dtype=torch.uint8, device="cuda")
    cache = prob.meta.get("cache")
    few_rows = Nq * (Hq // prob.Hkv) <= 32  # one row tile per key/value head: the library runs its decode kernel
    lens = None
    if cache:  # per-sequence lengths over a paged cache: fa_kvcache_fwd
        from paper_2307_08691_amd import inputs
        page = cache["page"]
        lens, table = inputs.cache_layout(cache["seed"], B, prob.Nk, page)
        pps = table.shape[1]
        tbl = torch.from_numpy(table).cuda()
        Kp, Vp = torch.empty((B * pps, page) + tuple(K.shape[2:]), dtype=K.dtype, device="cuda"), None
        Vp = torch.empty_like(Kp)
        Kp[tbl.long().flatten()] = K.view(B * pps, page, *K.shape[2:])  # (the drawn slabs, cut into pages)
        Vp[tbl.long().flatten()] = V.view(B * pps, page, *V.shape[2:])
        sl = torch.from_numpy(lens).cuda()
        del K, V

        def step():
            binding.fa_kvcache_fwd(Q, Kp, Vp, prob.scale, prob.causal, seqlens_k=sl, block_table=tbl, num_splits=splits,
                                   O=O, LSE=LSE, workspace=ws)
        kv_elems = 2.0 * float(lens.sum()) * prob.Hkv * d
    else:
        def step():
            binding.fa_splitkv_fwd(Q, K, V, prob.scale, prob.causal, splits, O=O, LSE=LSE, workspace=ws)
        kv_elems = float(K.numel() + V.numel())

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
    alg_bytes = 2.0 * (kv_elems + Q.numel() + O.numel()) + 4.0 * LSE.numel()
    gbs = alg_bytes / (kern_ms * 1e-3) / 1e9
    out = {
        "metric": "decode attention forward, GB/s of compulsory traffic (bf16)", "value": alg_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": prob.name, "B": B, "Nq": Nq, "Nk": prob.Nk, "Hq": Hq, "Hkv": prob.Hkv, "d": d,
                   "causal": prob.causal, "num_splits": splits, "algorithmic_bytes": alg_bytes,
                   **({"page": cache["page"], "cached_keys": int(lens.sum())} if cache else {})},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": 8000.0, "unit": "GB/s", "frac": gbs / 8000.0,
                     **traffic_fields(prob.name, "fwd_decode_kernel" if few_rows else "fwd_kernel"), "avg_kernel_ms": kern_ms,
                     "kernel": ("fwd_decode_kernel" if few_rows else "fwd_kernel<.., split>") + ("" if few_rows and splits == 1 else " + fwd_merge_kernel")},
    }
    if not args.no_cpu_baseline:
        from oracle import attention_oracle as orc
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < 10.0:
            b = n % B
            nk = prob.Nk if lens is None else int(lens[b])
            orc.attention_forward(orc.widen_bf16(prob.Q[b:b + 1]), orc.widen_bf16(prob.K[b:b + 1, :nk]),
                                  orc.widen_bf16(prob.V[b:b + 1, :nk]), prob.scale, prob.causal)
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
    ap.add_argument("--settle", type=float, default=0.25, metavar="SECONDS",
                    help="untimed work before the warm-up steps, so that the clocks have settled (0: none)")
    ap.add_argument("--workload", default="d128_n8k_causal")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fwd-only", action="store_true", help="profiling aid: a step is the forward alone")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the grid of section 4.1 and the other configs after the timed region")
    ap.add_argument("--list-workloads", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="profiling aid: instead of the benchmark, run 5 device-to-device copies of BYTES bytes; "
                         "under rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE they give the counters' scale factors")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    from paper_2307_08691_amd import inputs
    if args.list_workloads:
        print("\n".join(sorted(inputs.CONFIGS)))
        return 0
    import torch
    from paper_2307_08691_amd import binding

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
    if prob.dtype == "e4m3":
        return bench_fp8(args, prob, binding)
    if prob.Nk and not prob.varlen and prob.N * (prob.Hq // prob.Hkv) <= 256:
        return bench_decode(args, prob, binding)

    r = Runner(prob, binding, torch)
    step = r.fwd if args.fwd_only else r.both
    # A fresh process on an idle GPU first measures the clock ramp, not the kernels: a quarter of a
    # second of the same work, untimed, before the warm-up steps the caller asked for.
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # ---- the timed region: exactly `steps` steps of the entry points, nothing else
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    fwd_fl, bwd_fl = prob.fwd_flops(), prob.bwd_flops()
    total_fl = fwd_fl if args.fwd_only else fwd_fl + bwd_fl
    value = total_fl / (ms_per_step * 1e-3) / 1e12

    # ---- after it: the two passes apart, and each backward kernel on its own (HIP events)
    fwd_ms = r.event_ms(r.fwd, args.steps)
    bwd_ms = None if args.fwd_only else r.event_ms(r.bwd, args.steps)

    def roof(flops, ms, kernel):
        ach = flops / (ms * 1e-3) / 1e12
        return {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_BF16_TFLOPS, **traffic_fields(prob.name, kernel), "avg_kernel_ms": ms, "kernel": kernel}

    shape = {"T": prob.total_tokens, "nseq": len(prob.seqlens), "max_seqlen": int(prob.seqlens.max())} if prob.varlen else \
        {"B": prob.B, "N": prob.N, **({"Nk": prob.Nk} if prob.Nk else {})}
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
        "dtype": prob.dtype,  # the arithmetic type of the MFMA operands; accumulation is float32
        "data": "synthetic",
        "config": {"workload": prob.name, **shape, "Hq": prob.Hq, "Hkv": prob.Hkv, "d": prob.d, "causal": prob.causal,
                   "scale": prob.scale, "fwd_flops": fwd_fl, "bwd_flops": bwd_fl, "entry_points": r.entry_points(),
                   **{k: v for k, v in prob.meta.items() if k in ("dropout", "mask", "window", "block_pattern", "qk_mult")}},
        "frac_of_bf16_peak": value / PEAK_BF16_TFLOPS,
        "kernel_sources": kernel_sources_id(),
        "fwd": {"ms": fwd_ms, "tflops": fwd_fl / fwd_ms / 1e9, "frac_of_peak": fwd_fl / fwd_ms / 1e9 / PEAK_BF16_TFLOPS},
        "roofline_fwd": roof(fwd_fl, fwd_ms, "fwd_kernel"),
    }
    if bwd_ms is not None:
        out["bwd"] = {"ms": bwd_ms, "tflops": bwd_fl / bwd_ms / 1e9, "frac_of_peak": bwd_fl / bwd_ms / 1e9 / PEAK_BF16_TFLOPS}
    if args.fwd_only:
        out["roofline"] = out["roofline_fwd"]
    elif r.stages is not None:
        # metric FLOPs count 5 products (2.5 x forward); the dK/dV kernel performs 4 of them
        # (S, dP, dV, dK) and the dQ kernel 3 (S, dP recomputed, dQ): 2 x and 1.5 x forward
        prep_ms = r.event_ms(lambda: r.stages(1), args.steps)
        dkdv_ms = r.event_ms(lambda: r.stages(2), args.steps)
        dq_ms = r.event_ms(lambda: r.stages(4), args.steps)
        out["roofline"] = roof(2.0 * fwd_fl, dkdv_ms, "bwd_dkdv_kernel")
        out["roofline_dq"] = roof(1.5 * fwd_fl, dq_ms, "bwd_dq_kernel")
        out["bwd"]["prep_ms"] = prep_ms  # (a launch of its own only here: fa_bwd computes D inside the dQ kernel)
    else:
        # no per-kernel entry point for this workload: the backward launches together (with a D pre-pass
        # only at d = 256), against the 3.5 x forward FLOPs they execute (7 products)
        out["roofline"] = roof(3.5 * fwd_fl, bwd_ms, ("bwd_prep_kernel + " if prob.d == 256 else "") + "bwd_dkdv_kernel + bwd_dq_kernel")
    # what the matrix pipe sustains on this machine with every operand in registers (outside the timed region)
    out["mfma_loop"] = {}
    for key, rnd in (("constant_operands", False), ("random_operands", True)):
        tf, ghz = binding.fa_mfma_probe(2000, rnd)
        out["mfma_loop"][key] = {"tflops": tf, "shader_clock_ghz": ghz}
    if not args.no_sweep and not args.fwd_only and args.workload == "d128_n8k_causal":
        out["configs"] = {prob.name: three_rates(prob, fwd_ms, bwd_ms, ms_per_step)}
        out["configs"][prob.name]["entry_points"] = r.entry_points()
        del r
        for name in ("long_n16k_causal_x3", "gqa_ragged"):
            out["configs"][name] = measure_config(name, binding, torch, inputs)
        out["sweep"] = paper_grid(binding, torch, inputs)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(prob)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
