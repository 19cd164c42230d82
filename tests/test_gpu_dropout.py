"""GPU parity with dropout on P: fa_dropout_fwd / fa_dropout_bwd against the float64 oracle, which
regenerates the same keep mask from the same (seed, head, query, key) function. The mask decision
is integer arithmetic on both sides. The outputs carry the factor 1 / (1 - p), so what is asserted is
the yardstick clause: no worse than a bf16 implementation of the standard algorithm with the same
keep mask that materialises S and P (parity_util.judge with standard=False)."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402


def run(prob, p_drop, seed):
    Q, K, V, dO = (pu.to_gpu(x, prob.dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    O, L = binding.fa_dropout_fwd(Q, K, V, prob.scale, prob.causal, p_drop, seed)
    dQ, dK, dV = binding.fa_dropout_bwd(Q, K, V, O, dO, L, prob.scale, prob.causal, p_drop, seed)
    torch.cuda.synchronize()
    return dict(O=O, LSE=L, dQ=dQ, dK=dK, dV=dV)


def keep_masks(seed, p_drop, Hq):
    """keep_of(sequence, head, nq, nk) for parity_util.reference_batch, from the oracle's generator."""
    thr = orc.dropout_threshold(p_drop)
    return (lambda s, h, nq, nk: torch.from_numpy(orc.dropout_keep(seed, s * Hq + h, nq, nk, thr)).cuda()), 256.0 / (256.0 - thr)


def check_dropout(prob, p_drop, seed):
    got = run(prob, p_drop, seed)
    widen = orc.widen_f16 if prob.dtype == "f16" else orc.widen_bf16
    Q, K, V, dO = (widen(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    exp = {}
    exp["O"], exp["LSE"] = orc.attention_forward_dropout(Q, K, V, prob.scale, prob.causal, p_drop, seed)
    exp["dQ"], exp["dK"], exp["dV"] = orc.attention_backward_dropout(Q, K, V, dO, prob.scale, prob.causal, p_drop, seed)
    keep_of, rp = keep_masks(seed, p_drop, prob.Hq)
    ref = pu.reference_batch(*(pu.to_gpu(x, prob.dtype) for x in (prob.Q, prob.K, prob.V, prob.dO)), prob.scale,
                             prob.causal, keep_of=keep_of, rp=rp)
    res = pu.judge(f"dropout p={p_drop} {pu.describe(prob)}", {k: pu.to_f64(v) for k, v in got.items()}, exp, ref,
                   standard=False, dtype=prob.dtype, d=prob.d)
    return {k: v[0] for k, v in res.items()}


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("p_drop", [0.1, 0.5])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d", [(1, 1, 2, 2, 64), (65, 65, 2, 2, 64), (128, 128, 2, 2, 128), (257, 300, 4, 2, 128),
                                            (300, 515, 2, 1, 64), (33, 1000, 8, 2, 128)])
def test_dropout_matches_the_oracle(Nq, Nk, Hq, Hkv, d, p_drop, causal):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=6000 + Nq + Nk)
    check_dropout(prob, p_drop, seed=0x1234ABCD5678 + Nq)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d", [(65, 65, 2, 2, 64), (257, 300, 4, 2, 128), (300, 515, 2, 1, 64), (700, 700, 2, 2, 128)])
def test_dropout_in_half_precision(Nq, Nk, Hq, Hkv, d, causal):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=6050 + Nq + Nk, dtype="f16")
    check_dropout(prob, 0.25, seed=0x77AA11 + Nk)


def test_zero_probability_reproduces_the_plain_entry_points_bitwise():
    prob = inputs.make_cross(B=2, Nq=200, Nk=260, Hq=4, Hkv=2, d=128, causal=True, seed=6100)
    got = run(prob, 0.0, 42)
    ref = pu.run_hip(prob)
    for nm in got:
        assert torch.equal(got[nm], ref[nm]), nm


def test_lse_does_not_depend_on_the_mask_and_the_mask_depends_on_the_seed():
    prob = inputs.make_cross(B=1, Nq=129, Nk=129, Hq=2, Hkv=2, d=64, causal=False, seed=6200)
    a, b, plain = run(prob, 0.25, 1), run(prob, 0.25, 2), pu.run_hip(prob)
    assert torch.equal(a["LSE"], plain["LSE"]) and torch.equal(b["LSE"], plain["LSE"])
    assert not torch.equal(a["O"], b["O"])
    again = run(prob, 0.25, 1)
    for nm in a:
        assert torch.equal(a[nm], again[nm]), nm  # same seed, same bits


def test_kept_fraction_seen_through_the_output():
    """V = all ones: every output element is (number of kept keys) / ((1 - p) Nk) for uniform P."""
    B, N, H, d = 1, 512, 2, 64
    Q = torch.zeros(B, N, H, d, dtype=torch.bfloat16, device="cuda")  # uniform probabilities
    K = torch.zeros_like(Q)
    V = torch.ones_like(Q)
    O, _ = binding.fa_dropout_fwd(Q, K, V, 0.125, False, 0.25, 7)
    torch.cuda.synchronize()
    thr = orc.dropout_threshold(0.25)
    for h in range(H):
        keep = orc.dropout_keep(7, h, N, N, thr)
        want = keep.sum(axis=1) / (0.75 * N)
        assert np.max(np.abs(pu.to_f64(O[0, :, h, 0]) - want)) <= 2 * pu.bf16_ulp(float(want.max()))


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("d,Hq,Hkv", [(64, 2, 2), (128, 4, 2)])
def test_ragged_batches_with_dropout(d, Hq, Hkv, causal, dtype):
    """fa_varlen_dropout_fwd / bwd against the oracle's ragged dropout: the generator counts rows and
    columns from the start of each sequence and uses sequence * Hq + head as its head index."""
    prob = inputs.make_varlen([100, 257, 1, 31, 300], Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=6100 + d, dtype=dtype)
    Q, K, V, dO = (pu.to_gpu(x, dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    cu = torch.from_numpy(prob.cu_seqlens.astype(np.int32)).cuda()
    p_drop, seed = 0.25, 0x1234567890ABCDEF
    O, L = binding.fa_varlen_dropout_fwd(Q, K, V, cu, 300, prob.scale, causal, p_drop, seed)
    dQ, dK, dV = binding.fa_varlen_dropout_bwd(Q, K, V, O, dO, L, cu, 300, prob.scale, causal, p_drop, seed)
    torch.cuda.synchronize()
    widen = orc.widen_f16 if dtype == "f16" else orc.widen_bf16
    Qf, Kf, Vf, dOf = (widen(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    eO, eL = orc.varlen_forward_dropout(Qf, Kf, Vf, prob.cu_seqlens, prob.scale, causal, p_drop, seed)
    edQ, edK, edV = orc.varlen_backward_dropout(Qf, Kf, Vf, dOf, prob.cu_seqlens, prob.scale, causal, p_drop, seed)
    keep_of, rp = keep_masks(seed, p_drop, Hq)
    ref = pu.reference_batch(Q, K, V, dO, prob.scale, causal, cu_q=prob.cu_seqlens, keep_of=keep_of, rp=rp)
    pu.judge(f"ragged dropout d{d} H{Hq}/{Hkv} causal={causal}",
             {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))},
             dict(O=eO, LSE=eL, dQ=edQ, dK=edK, dV=edV), ref, standard=False, dtype=dtype, d=d)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["dropout_d128_n8k_causal", "dropout_gqa_ragged"])
def test_full_size_dropout_workloads_sampled_units(name):
    """The benchmark shapes with dropout (p = 0.1): whole (sequence, head) units against the oracle
    and the 16-bit reference with the same keep mask; the ragged one on its shortest and longest
    sequence (grouped heads: dK, dV of a key/value head over its four query heads)."""
    prob = inputs.make_config(name)
    p_drop, seed = prob.meta["dropout"]
    thr = orc.dropout_threshold(p_drop)
    rp = 256.0 / (256.0 - thr)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    G = prob.Hq // prob.Hkv
    if prob.varlen:
        cu = torch.from_numpy(prob.cu_seqlens.astype(np.int32)).cuda()
        mx = int(prob.seqlens.max())
        O, L = binding.fa_varlen_dropout_fwd(Q, K, V, cu, mx, prob.scale, True, p_drop, seed)
        dQ, dK, dV = binding.fa_varlen_dropout_bwd(Q, K, V, O, dO, L, cu, mx, prob.scale, True, p_drop, seed)
        units = [(s, s % prob.Hkv, int(prob.cu_seqlens[s]), int(prob.cu_seqlens[s + 1]))
                 for s in sorted({int(np.argmin(prob.seqlens)), int(np.argmax(prob.seqlens))})]
    else:
        O, L = binding.fa_dropout_fwd(Q, K, V, prob.scale, True, p_drop, seed)
        dQ, dK, dV = binding.fa_dropout_bwd(Q, K, V, O, dO, L, prob.scale, True, p_drop, seed)
        units = [(0, 0, 0, prob.N), (prob.B - 1, prob.Hkv - 1, 0, prob.N)]
    torch.cuda.synchronize()
    for t in (O, L, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()
    for (s, g, a, e) in units:
        n = e - a
        sel = (slice(a, e),) if prob.varlen else (s,)
        k, v = orc.widen_bf16(prob.K[sel][:, g]), orc.widen_bf16(prob.V[sel][:, g])
        exp = {"O": [], "LSE": [], "dQ": [], "dK": np.zeros_like(k), "dV": np.zeros_like(v)}
        ref = {"O": [], "LSE": [], "dQ": [], "dK": np.zeros_like(k), "dV": np.zeros_like(v)}
        for h in range(g * G, (g + 1) * G):
            keep = orc.dropout_keep(seed, s * prob.Hq + h, n, n, thr)
            q, do = orc.widen_bf16(prob.Q[sel][:, h]), orc.widen_bf16(prob.dO[sel][:, h])
            o, lse, _ = orc.head_forward_dropout(q, k, v, prob.scale, True, keep, thr)
            dq, dk, dv = orc.head_backward_dropout(q, k, v, do, prob.scale, True, keep, thr)
            r = pu.reference_head(Q[sel][:, h], K[sel][:, g], V[sel][:, g], dO[sel][:, h], prob.scale, True,
                                  keep=torch.from_numpy(keep).cuda(), rp=rp)
            for nm, x in (("O", o), ("LSE", lse), ("dQ", dq)):
                exp[nm].append(x)
                ref[nm].append(r[nm])
            exp["dK"] += dk
            exp["dV"] += dv
            ref["dK"] += r["dK"]
            ref["dV"] += r["dV"]
        hs = slice(g * G, (g + 1) * G)
        got = {"O": pu.to_f64(O[sel][:, hs]).transpose(1, 0, 2), "LSE": pu.to_f64(L[hs, a:e] if prob.varlen else L[s, hs]),
               "dQ": pu.to_f64(dQ[sel][:, hs]).transpose(1, 0, 2), "dK": pu.to_f64(dK[sel][:, g]), "dV": pu.to_f64(dV[sel][:, g])}
        for nm in ("O", "LSE", "dQ"):
            exp[nm], ref[nm] = np.stack(exp[nm]), np.stack(ref[nm])
        pu.judge(f"{name} unit (s={s}, g={g}, n={n})", got, exp, ref, standard=False, d=prob.d)
