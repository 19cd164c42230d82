"""Helpers for the GPU parity tests: move seeded 16-bit patterns to the GPU, run the HIP
path through the C ABI binding, run the float64 oracle on the same bits, build the 16-bit
"materialising" reference, and judge the three against each other. Test-side only.

What is asserted, by `judge` (every GPU parity test ends there):

  1. inputs drawn from N(0,1) without dropout (`standard`): the fixed bounds against the
     float64 oracle, |dO| <= 2e-2, |d(dQ, dK, dV)| <= 5e-2, |dLSE| <= 1e-3, on every element.
     One exception, decided per element from the exact value alone: where the element type
     cannot represent the exact value to within the bound (half its spacing at that value
     exceeds the bound: bfloat16 values of magnitude 16 and above for 5e-2), the element must
     be within that half spacing instead, i.e. be a correct rounding up to the bound. Only
     degenerate shapes reach such magnitudes with N(0,1) inputs (one key and hundreds of
     queries: dV is a sum of hundreds of dO rows);
  2. every case: the HIP path is no worse than a 16-bit implementation of section 2.2's
     standard algorithm that materialises S and P in the element type (`reference_head`):
     err_hip <= err_reference + one unit in the last place of the element type at the tensor's
     largest magnitude (the slack the comparison was specified with before any kernel
     existed; both implementations round their operands and their result, so their worst
     elements differ by chance by about that much);
  3. inputs that are scaled up, or dropout (outputs scaled by 1/(1-p)): clause 2 alone decides
     for O, dQ, dK, dV; whether the fixed bounds happen to hold is printed, not asserted.
     LSE, a float32 output, keeps 1e-3 up to the point where float32 accumulation of the d
     products of a score can exceed it: max(1e-3, d * 2^-24 * max|LSE|).

No bound here is a multiple fitted to a measurement.
"""
from __future__ import annotations

import math
import os

import numpy as np

from oracle import attention_oracle as orc
from paper_2307_08691_amd import binding
from paper_2307_08691_amd.inputs import AttnProblem

# Absolute bounds against the float64 oracle for 16-bit inputs drawn from N(0,1).
TOL_O = 2e-2
TOL_GRAD = 5e-2
TOL_LSE = 1e-3
FIXED = {"O": TOL_O, "LSE": TOL_LSE, "dQ": TOL_GRAD, "dK": TOL_GRAD, "dV": TOL_GRAD, "dM": TOL_GRAD}


def to_gpu(bits: np.ndarray, dtype: str = "bf16"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(
        torch.float16 if dtype == "f16" else torch.bfloat16)


def to_f64(t) -> np.ndarray:
    return t.detach().double().cpu().numpy()


def ulp(maxabs: float, dtype: str = "bf16") -> float:
    """Spacing of the element type's numbers at magnitude `maxabs`: bfloat16 has 8 significand
    bits, IEEE half precision 11 (and nothing finer than 2^-24)."""
    if maxabs <= 0:
        return 0.0
    e = math.floor(math.log2(maxabs))
    return 2.0 ** (e - 7) if dtype == "bf16" else 2.0 ** (max(e, -14) - 10)


def bf16_ulp(maxabs: float) -> float:
    return ulp(maxabs, "bf16")


def half_spacing(x: np.ndarray, dtype: str = "bf16") -> np.ndarray:
    """Elementwise: half the spacing of the element type's numbers at |x| (0 at 0)."""
    a = np.abs(np.asarray(x, dtype=np.float64))
    e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    sp = np.exp2(e - 7) if dtype == "bf16" else np.exp2(np.maximum(e, -14) - 10)
    return np.where(a > 0, 0.5 * sp, 0.0)


def maxdiff(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.max(np.abs(a - b))) if a.size else 0.0


def maxabs(a: np.ndarray) -> float:
    a = np.asarray(a)
    a = a[np.isfinite(a)]
    return float(np.max(np.abs(a))) if a.size else 0.0


# ---------------------------------------------------------------------------------------------
# the 16-bit yardstick
# ---------------------------------------------------------------------------------------------

def reference_head(q, k, v, do, scale, causal, M=None, keep=None, rp=1.0, backward=True, pos=None):
    """The 'standard implementation' of section 2.2 in the element type of `q` (bfloat16 or
    half precision): matmuls on 16-bit tensors, S and P stored in 16 bits, softmax in float32.
    One head, torch on the GPU. `M` [Nq, Nk]: additive mask (finite or -inf); `keep` [Nq, Nk]
    bool with rp = 1 / (1 - p): dropout on P. `pos` (sampled query rows of a longer sequence): the
    rows' positions among the keys for the causal rule; dK, dV are then partial sums over those
    rows only. Returns float64 numpy arrays O, LSE and (backward) dQ, dK, dV. Test-side yardstick
    only: the HIP path must not be less accurate than this."""
    import torch
    et = q.dtype
    s32 = (q @ k.T).float() * scale
    if M is not None:
        s32 = s32 + M.float()
    sf = s32.to(et).float()  # S as stored
    del s32
    if causal:
        n, nk = q.shape[0], k.shape[0]
        if pos is None:
            hidden = torch.ones(n, nk, dtype=torch.bool, device=q.device).triu(1 + nk - n)
        else:
            hidden = torch.arange(nk, device=q.device)[None, :] > torch.as_tensor(pos, device=q.device)[:, None]
        sf = sf.masked_fill(hidden, float("-inf"))
        del hidden
    lse = torch.logsumexp(sf, dim=-1)
    p32 = torch.exp(sf - torch.where(torch.isneginf(lse), torch.zeros_like(lse), lse)[:, None])  # rows without keys: 0
    del sf
    p = p32.to(et)  # P as stored
    del p32
    pd = p if keep is None else (p.float() * keep * rp).to(et)
    o = pd @ v
    out = {"O": to_f64(o), "LSE": to_f64(lse)}
    if backward:
        out["dV"] = to_f64(pd.T @ do)
        dp = (do @ v.T).float()
        if keep is not None:
            dp = dp * keep * rp
        big_d = (do.float() * o.float()).sum(dim=-1, keepdim=True)
        ds = (p.float() * (dp - big_d)).to(et)
        del dp
        out["dM"] = ds  # (left on the GPU: only the mask-gradient tests fetch it)
        out["dQ"] = to_f64(((ds @ k).float() * scale).to(et))
        out["dK"] = to_f64(((ds.T @ q).float() * scale).to(et))
    return out


# ---------------------------------------------------------------------------------------------
# the judgement
# ---------------------------------------------------------------------------------------------

_REPORT = os.environ.get("FA_PARITY_REPORT")  # optional: append one line per judged tensor to this file


def judge(label, got, exp, ref, *, standard=True, dtype="bf16", d=128):
    """got, exp, ref: name -> float64 arrays of equal shapes (names among O, LSE, dQ, dK, dV).
    LSE may hold -inf (rows without keys): the places must agree and are left out of the
    comparison. Asserts the clauses of this module's header; returns name -> (error, error in
    units of the last place, reference error)."""
    res = {}
    lines = []
    failures = []
    for nm in got:
        g, e = np.asarray(got[nm], dtype=np.float64), np.asarray(exp[nm], dtype=np.float64)
        assert g.shape == e.shape, f"{label}: {nm} shape {g.shape} against {e.shape}"
        r = None if ref is None or nm not in ref else np.asarray(ref[nm], dtype=np.float64)
        if nm == "LSE":
            dead = np.isneginf(e)
            assert np.array_equal(np.isneginf(g), dead), f"{label}: rows without keys differ in LSE"
            g, e = np.where(dead, 0.0, g), np.where(dead, 0.0, e)
            if r is not None:
                r = np.where(dead, 0.0, r)
        assert np.all(np.isfinite(g)), f"{label}: {nm} has non-finite values"
        err, mag = maxdiff(g, e), maxabs(e)
        u = ulp(mag, dtype)
        ref_err = None if r is None else maxdiff(r, e)
        if nm == "LSE":
            bound = TOL_LSE if standard else max(TOL_LSE, d * 2.0 ** -24 * mag)
            if err > bound:
                failures.append(f"{nm} err {err:.3e} > {bound:.3e}")
        else:
            if standard and err > FIXED[nm]:
                over = np.abs(g - e) - np.maximum(FIXED[nm], half_spacing(e, dtype))
                if np.any(over > 0):
                    failures.append(f"{nm} err {err:.3e} > fixed bound {FIXED[nm]:.0e} (max|.| {mag:.3g}, {err / u if u else 0:.2f} ulp)")
            assert ref_err is not None, f"{label}: no 16-bit reference for {nm}"
            if err > ref_err + u:
                failures.append(f"{nm} err {err:.3e} ({err / u if u else 0:.2f} ulp) worse than the 16-bit reference "
                                f"{ref_err:.3e} + one ulp {u:.3e}")
        res[nm] = (err, err / u if u else 0.0, ref_err)
        lines.append(f"{label:60s} {nm:3s} err {err:9.3e} = {err / u if u else 0:6.2f} ulp  ref "
                     f"{'-' if ref_err is None else format(ref_err, '9.3e')}  max|.| {mag:8.3g}  "
                     f"{'standard' if standard else 'scaled  '} meets_fixed={err <= FIXED[nm]}")
    print("\n".join(lines))
    if _REPORT:
        with open(_REPORT, "a") as f:
            f.write("\n".join(lines) + "\n")
    assert not failures, f"{label}: " + "; ".join(failures)
    return res


def is_standard(prob: AttnProblem) -> bool:
    return bool(prob.meta.get("standard_normal", True))


# ---------------------------------------------------------------------------------------------
# HIP path, oracle, reference on a whole problem
# ---------------------------------------------------------------------------------------------

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


def reference_batch(Q, K, V, dO, scale, causal, backward=True, cu_q=None, cu_k=None, M=None, keep_of=None, rp=1.0,
                    M_of=None, want_dm=False):
    """The 16-bit reference over a whole batch, in the oracle's layouts. Q, K, V, dO: torch tensors
    on the GPU, dense [B, N, H, d] or packed [T, H, d] with cumulative offsets cu_q (and cu_k for
    two lengths). M: torch [Bm, Hm, Nq, Nk] or None (dense only), or M_of(seq, head, nq, nk) ->
    torch [nq, nk]. keep_of(seq, head, nq, nk) -> torch bool [nq, nk] or None. dK, dV of grouped
    heads are summed in float64."""
    packed = cu_q is not None
    Hq, Hkv = Q.shape[-2], K.shape[-2]
    G = Hq // Hkv
    if packed:
        cu_k = cu_q if cu_k is None else cu_k
        nseq = len(cu_q) - 1
        out = {"O": np.zeros(tuple(Q.shape)), "LSE": np.zeros((Hq, Q.shape[0]))}
    else:
        nseq = Q.shape[0]
        out = {"O": np.zeros(tuple(Q.shape)), "LSE": np.zeros((nseq, Hq, Q.shape[1]))}
    if backward:
        out.update(dQ=np.zeros(tuple(Q.shape)), dK=np.zeros(tuple(K.shape)), dV=np.zeros(tuple(V.shape)))
    if want_dm:  # dense only: the 16-bit dS of every (sequence, head)
        out["dM"] = np.zeros((nseq, Hq, Q.shape[1], K.shape[1]))
    for s in range(nseq):
        if packed:
            a, e, ak, ek = int(cu_q[s]), int(cu_q[s + 1]), int(cu_k[s]), int(cu_k[s + 1])
            if e == a or ek == ak:  # (a sequence without keys has no softmax to materialise: zeros)
                continue
            qs, ks, vs, gs = Q[a:e], K[ak:ek], V[ak:ek], dO[a:e]
        else:
            qs, ks, vs, gs = Q[s], K[s], V[s], dO[s]
        for h in range(Hq):
            m = None if M is None else M[s if M.shape[0] > 1 else 0, h if M.shape[1] > 1 else 0]
            if M_of is not None:
                m = M_of(s, h, qs.shape[0], ks.shape[0])
            keep = None if keep_of is None else keep_of(s, h, qs.shape[0], ks.shape[0])
            r = reference_head(qs[:, h], ks[:, h // G], vs[:, h // G], gs[:, h], scale, causal, M=m, keep=keep, rp=rp,
                               backward=backward)
            if packed:
                out["O"][a:e, h] = r["O"]
                out["LSE"][h, a:e] = r["LSE"]
                if backward:
                    out["dQ"][a:e, h] = r["dQ"]
                    out["dK"][ak:ek, h // G] += r["dK"]
                    out["dV"][ak:ek, h // G] += r["dV"]
            else:
                out["O"][s, :, h] = r["O"]
                out["LSE"][s, h] = r["LSE"]
                if backward:
                    out["dQ"][s, :, h] = r["dQ"]
                    out["dK"][s, :, h // G] += r["dK"]
                    out["dV"][s, :, h // G] += r["dV"]
                if want_dm:
                    out["dM"][s, h] = to_f64(r["dM"])
    return out


def run_reference(prob: AttnProblem, backward: bool = True):
    Q, K, V, dO = (to_gpu(x, prob.dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    return reference_batch(Q, K, V, dO, prob.scale, prob.causal, backward,
                           cu_q=prob.cu_seqlens if prob.varlen else None)


def check(prob: AttnProblem, backward: bool = True):
    """HIP path against oracle and reference on every element of a (small) problem."""
    got = {k: to_f64(v) for k, v in run_hip(prob, backward).items()}
    res = judge(prob.name + f" {describe(prob)}", got, run_oracle(prob, backward), run_reference(prob, backward),
                standard=is_standard(prob), dtype=prob.dtype, d=prob.d)
    return {k: v[0] for k, v in res.items()}


def describe(prob: AttnProblem) -> str:
    if prob.varlen:
        return f"ragged{list(map(int, prob.seqlens))} H{prob.Hq}/{prob.Hkv} d{prob.d} {'c' if prob.causal else 'f'} {prob.dtype}"
    return f"B{prob.B} N{prob.N}x{prob.keys} H{prob.Hq}/{prob.Hkv} d{prob.d} {'c' if prob.causal else 'f'} {prob.dtype}"


def check_units(prob: AttnProblem, got, units):
    """Full-size dense problems: whole (sequence b, key/value head g) units, every query head of
    the group, against oracle and reference. got: torch tensors from run_hip."""
    G = prob.Hq // prob.Hkv
    widen = orc.widen_f16 if prob.dtype == "f16" else orc.widen_bf16
    Qg, Kg, Vg, dOg = (to_gpu(x, prob.dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    worst = {}
    for (b, g) in units:
        k, v = widen(prob.K[b, :, g]), widen(prob.V[b, :, g])
        exp = {nm: [] for nm in ("O", "LSE", "dQ")}
        ref = {nm: [] for nm in ("O", "LSE", "dQ")}
        exp["dK"], exp["dV"] = np.zeros_like(k), np.zeros_like(v)
        ref["dK"], ref["dV"] = np.zeros_like(k), np.zeros_like(v)
        for h in range(g * G, (g + 1) * G):
            q, do = widen(prob.Q[b, :, h]), widen(prob.dO[b, :, h])
            o, lse, _ = orc.head_forward(q, k, v, prob.scale, prob.causal)
            dq, dk, dv = orc.head_backward(q, k, v, do, prob.scale, prob.causal)
            r = reference_head(Qg[b, :, h], Kg[b, :, g], Vg[b, :, g], dOg[b, :, h], prob.scale, prob.causal)
            for nm, e in (("O", o), ("LSE", lse), ("dQ", dq)):
                exp[nm].append(e)
                ref[nm].append(r[nm])
            exp["dK"] += dk
            exp["dV"] += dv
            ref["dK"] += r["dK"]
            ref["dV"] += r["dV"]
        hs = slice(g * G, (g + 1) * G)
        gotu = {"O": to_f64(got["O"][b, :, hs]).transpose(1, 0, 2), "LSE": to_f64(got["LSE"][b, hs]),
                "dQ": to_f64(got["dQ"][b, :, hs]).transpose(1, 0, 2), "dK": to_f64(got["dK"][b, :, g]),
                "dV": to_f64(got["dV"][b, :, g])}
        for nm in ("O", "LSE", "dQ"):
            exp[nm], ref[nm] = np.stack(exp[nm]), np.stack(ref[nm])
        res = judge(f"{prob.name} unit (b={b}, g={g})", gotu, exp, ref, standard=is_standard(prob), dtype=prob.dtype,
                    d=prob.d)
        for nm, (err, _, _) in res.items():
            worst[nm] = max(worst.get(nm, 0.0), err)
    return worst
