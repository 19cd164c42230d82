"""Helpers for the GPU parity tests: move seeded bf16 bit patterns to the GPU,
run the HIP path through the C ABI binding, run the float64 oracle on the same
bits, and build the bf16 "materialising" reference the tolerances are judged
against. Test-side only."""
from __future__ import annotations

import math

import numpy as np

from oracle import attention_oracle as orc
from paper_2307_08691_amd import binding
from paper_2307_08691_amd.inputs import AttnProblem

# Absolute bounds against the float64 oracle for bf16 inputs drawn from N(0,1).
TOL_O = 2e-2
TOL_GRAD = 5e-2
TOL_LSE = 1e-3


def tolerance(name: str, expected: np.ndarray) -> float:
    """Absolute bound on max|HIP - oracle| for one output tensor.

    The stated bounds (2e-2 on O, 5e-2 on gradients, 1e-3 on LSE) hold for
    N(0,1) inputs, where outputs stay below about 8 in magnitude. Outputs are
    stored in bf16, so rounding the exact result alone costs half a bf16 ulp
    (2^-9 relative): for inputs scaled up (the x3 stress workload, gradients
    beyond 10) no bf16 output can meet a fixed 5e-2. The bound therefore
    never drops below 2 ulp at the tensor's largest magnitude: half an ulp for
    the final rounding, the rest for the bf16 rounding of the P and dS
    operands of the second-stage products (2^-9 relative per term), which for
    the peaked softmax of the stress workload is carried by a few dominant
    terms and does not average out (measured: up to 1.6 ulp at N = 16384; a
    bf16 implementation that materialises S and P is off by more than 10 ulp
    there)."""
    base = {"O": TOL_O, "LSE": TOL_LSE}.get(name, TOL_GRAD)
    if name == "LSE":
        return base
    return max(base, 2.0 * bf16_ulp(float(np.max(np.abs(expected))) if expected.size else 0.0))


def to_gpu(bits: np.ndarray, dtype: str = "bf16"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(
        torch.float16 if dtype == "f16" else torch.bfloat16)


def to_f64(t) -> np.ndarray:
    return t.detach().double().cpu().numpy()


def bf16_ulp(maxabs: float) -> float:
    """Spacing of bfloat16 numbers at magnitude `maxabs` (8 significand bits)."""
    if maxabs <= 0:
        return 0.0
    return 2.0 ** (math.floor(math.log2(maxabs)) - 7)


def run_hip(prob: AttnProblem, backward: bool = True):
    """Run the HIP path. Returns dict of torch tensors (O, LSE, dQ, dK, dV)."""
    import torch
    Q, K, V, dO = (to_gpu(x, prob.dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    out = {}
    if prob.varlen:
        cu = torch.from_numpy(prob.cu_seqlens.astype(np.int32)).cuda()
        mx = int(prob.seqlens.max())
        O, LSE = binding.fa_varlen_fwd(Q, K, V, cu, mx, prob.scale, prob.causal)
        out.update(O=O, LSE=LSE)
        if backward:
            dQ, dK, dV = binding.fa_varlen_bwd(Q, K, V, O, dO, LSE, cu, mx, prob.scale, prob.causal)
            out.update(dQ=dQ, dK=dK, dV=dV)
    elif prob.Nk:
        O, LSE = binding.fa_cross_fwd(Q, K, V, prob.scale, prob.causal)
        out.update(O=O, LSE=LSE)
        if backward:
            dQ, dK, dV = binding.fa_cross_bwd(Q, K, V, O, dO, LSE, prob.scale, prob.causal)
            out.update(dQ=dQ, dK=dK, dV=dV)
    else:
        O, LSE = binding.fa_fwd(Q, K, V, prob.scale, prob.causal)
        out.update(O=O, LSE=LSE)
        if backward:
            dQ, dK, dV = binding.fa_bwd(Q, K, V, O, dO, LSE, prob.scale, prob.causal)
            out.update(dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    return out


def run_oracle(prob: AttnProblem, backward: bool = True):
    widen = orc.widen_f16 if prob.dtype == "f16" else orc.widen_bf16
    Q, K, V, dO = (widen(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    out = {}
    if prob.varlen:
        out["O"], out["LSE"] = orc.varlen_forward(Q, K, V, prob.cu_seqlens, prob.scale, prob.causal)
        if backward:
            out["dQ"], out["dK"], out["dV"] = orc.varlen_backward(Q, K, V, dO, prob.cu_seqlens, prob.scale, prob.causal)
    else:
        out["O"], out["LSE"] = orc.attention_forward(Q, K, V, prob.scale, prob.causal)
        if backward:
            out["dQ"], out["dK"], out["dV"] = orc.attention_backward(Q, K, V, dO, prob.scale, prob.causal)
    return out


def bf16_reference_head(q, k, v, do, scale, causal):
    """The 'standard implementation' of section 2.2 in bf16: matmuls on bf16
    tensors, S and P stored as bf16, softmax in fp32. One head, torch on the
    GPU. Returns O, dQ, dK, dV as float64 numpy arrays. Test-side yardstick
    only: the HIP path must not be less accurate than this."""
    import torch
    bf = q.dtype  # bfloat16 or float16: the element type under test
    s = ((q @ k.T).float() * scale).to(bf)
    sf = s.float()
    if causal:
        n, nk = q.shape[0], k.shape[0]
        mask = torch.ones(n, nk, dtype=torch.bool, device=q.device).triu(1 + nk - n)
        sf = sf.masked_fill(mask, float("-inf"))
    p32 = torch.softmax(sf, dim=-1)
    p = p32.to(bf)
    o = p @ v
    dv = p.T @ do
    dp = (do @ v.T).float()
    big_d = (do.float() * o.float()).sum(dim=-1, keepdim=True)
    ds = (p.float() * (dp - big_d)).to(bf)
    dq = ((ds @ k).float() * scale).to(bf)
    dk = ((ds.T @ q).float() * scale).to(bf)
    return tuple(to_f64(x) for x in (o, dq, dk, dv))


def maxdiff(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.max(np.abs(a - b))) if a.size else 0.0
