"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times. The float64 oracle cannot materialise every (sequence, head) unit of
these workloads in seconds, so whole units are sampled (first and last head,
first and last sequence; shortest and longest sequence of the ragged batch) and
compared element by element; everything else is checked through properties that
hold at any size (finiteness, dV column sums)."""
import numpy as np
import pytest

from paper_2307_08691_amd import inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402


def check_units(prob, got, units):
    """units: list of (b, kv_head). Compares O, LSE, dQ for every query head of
    the group and dK, dV of the kv head."""
    G = prob.Hq // prob.Hkv
    widen = orc.widen_f16 if prob.dtype == "f16" else orc.widen_bf16
    worst = {}
    for (b, g) in units:
        k = widen(prob.K[b, :, g])
        v = widen(prob.V[b, :, g])
        dk_sum = np.zeros_like(k)
        dv_sum = np.zeros_like(v)
        for h in range(g * G, (g + 1) * G):
            q = widen(prob.Q[b, :, h])
            do = widen(prob.dO[b, :, h])
            o, lse, _ = orc.head_forward(q, k, v, prob.scale, prob.causal)
            dq, dk, dv = orc.head_backward(q, k, v, do, prob.scale, prob.causal)
            dk_sum += dk
            dv_sum += dv
            for nm, e, gt in (("O", o, got["O"][b, :, h]), ("LSE", lse, got["LSE"][b, h]), ("dQ", dq, got["dQ"][b, :, h])):
                err = pu.maxdiff(pu.to_f64(gt), e)
                tol = pu.tolerance(nm, e)
                assert err <= tol, f"{prob.name} unit (b={b}, h={h}): {nm} err {err:.3e} > {tol:.3e}"
                worst[nm] = max(worst.get(nm, 0.0), err)
        for nm, e, gt in (("dK", dk_sum, got["dK"][b, :, g]), ("dV", dv_sum, got["dV"][b, :, g])):
            err = pu.maxdiff(pu.to_f64(gt), e)
            tol = pu.tolerance(nm, e)
            assert err <= tol, f"{prob.name} unit (b={b}, g={g}): {nm} err {err:.3e} > {tol:.3e}"
            worst[nm] = max(worst.get(nm, 0.0), err)
    return worst


def global_properties(prob, got):
    for nm, t in got.items():
        assert torch.isfinite(t.float()).all(), f"{prob.name}: {nm} not finite"
    if not prob.varlen and prob.Hq == prob.Hkv:
        # rows of P sum to one => per (batch, head) the columns of dV sum to those of dO
        dO = pu.to_gpu(prob.dO).double().sum(dim=1)
        dV = got["dV"].double().sum(dim=1)
        scale = float(pu.to_gpu(prob.dO).double().abs().sum(dim=1).max())
        assert float((dO - dV).abs().max()) <= 4e-3 * scale


@pytest.mark.parametrize("name", ["d128_n8k_causal", "sweep_d64_n8192_full", "sweep_d64_n2048_causal",
                                  "sweep_d128_n512_full", "d96_n8k_causal", "d32_n8k_causal", "d256_n8k_causal"])
def test_dense_workloads_sampled_units(name):
    prob = inputs.make_config(name)
    got = pu.run_hip(prob)
    global_properties(prob, got)
    units = [(0, 0), (prob.B - 1, prob.Hkv - 1)]
    print(name, check_units(prob, got, units))


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Nq,Nk,Hq,Hkv", [(4, 512, 512, 64, 64), (2, 1000, 1000, 64, 16), (8, 512, 512, 64, 8),
                                            (16, 300, 300, 64, 64), (2, 1024, 1024, 64, 64), (4, 512, 777, 64, 16)])
def test_short_sequences_in_chained_workgroups(B, Nq, Nk, Hq, Hkv, causal, dtype):
    """Dense d = 128 batches of short sequences whose forward pass runs in workgroups that take
    2, 4 or 8 (row block, head, sequence) items in a row, fetching an item's Q_i and first tiles
    while the previous one finishes: units from both ends and the middle of the batch, which sit
    at different places of different chains; ragged last row blocks (N = 1000, 300); more keys
    than queries."""
    prob = inputs.make_cross(B=B, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=128, causal=causal, seed=15000 + Nq + Hkv, dtype=dtype)
    got = pu.run_hip(prob)
    for nm, t in got.items():
        assert torch.isfinite(t.float()).all(), nm
    units = [(0, 0), (B // 2, Hkv // 2), (B - 1, Hkv - 1), (B - 1, 0), (0, Hkv - 1)]
    print(prob.name, check_units(prob, got, units))


def test_long_context_wide_range_sampled_units():
    prob = inputs.make_config("long_n16k_causal_x3")
    got = pu.run_hip(prob)
    global_properties(prob, got)
    print(prob.name, check_units(prob, got, [(0, 15)]))
    # sampled rows of another head, forward only (cheap: one row block of scores at a time)
    rows = np.asarray([0, 1, 127, 128, 8191, 8192, 16000, 16383])
    k = orc.widen_bf16(prob.K[0, :, 3])
    v = orc.widen_bf16(prob.V[0, :, 3])
    q = orc.widen_bf16(prob.Q[0, rows, 3])
    o, lse = orc.rows_forward(q, rows, k, v, prob.scale, True)
    assert pu.maxdiff(pu.to_f64(got["O"][0, rows, 3]), o) <= pu.tolerance("O", o)
    assert pu.maxdiff(pu.to_f64(got["LSE"][0, 3, rows]), lse) <= pu.TOL_LSE


def test_gqa_ragged_sampled_sequences():
    prob = inputs.make_config("gqa_ragged")
    got = pu.run_hip(prob)
    for nm, t in got.items():
        assert torch.isfinite(t.float()).all(), nm
    lens = prob.seqlens
    cu = prob.cu_seqlens
    picks = sorted({int(np.argmin(lens)), int(np.argmax(lens)), 0, len(lens) - 1})
    G = prob.Hq // prob.Hkv
    for s in picks:
        a, e = int(cu[s]), int(cu[s + 1])
        g = s % prob.Hkv
        hs = slice(g * G, (g + 1) * G)
        Q = orc.widen_bf16(prob.Q[a:e, hs])[None]
        dO = orc.widen_bf16(prob.dO[a:e, hs])[None]
        K = orc.widen_bf16(prob.K[a:e, g:g + 1])[None]
        V = orc.widen_bf16(prob.V[a:e, g:g + 1])[None]
        O, L = orc.attention_forward(Q, K, V, prob.scale, True)
        dQ, dK, dV = orc.attention_backward(Q, K, V, dO, prob.scale, True)
        for nm, exp, gt in (("O", O[0], got["O"][a:e, hs]), ("LSE", L[0], got["LSE"][hs, a:e]),
                            ("dQ", dQ[0], got["dQ"][a:e, hs]), ("dK", dK[0], got["dK"][a:e, g:g + 1]),
                            ("dV", dV[0], got["dV"][a:e, g:g + 1])):
            err = pu.maxdiff(pu.to_f64(gt), exp)
            tol = pu.tolerance(nm, exp)
            assert err <= tol, f"ragged seq {s} (len {e - a}) kv head {g}: {nm} err {err:.3e} > {tol:.3e}"


@pytest.mark.timeout(900)
def test_tensors_beyond_two_to_the_31_elements():
    """Maximum sizes: 4 x 32768 x 128 heads x 128 = 2^31 elements (4 GiB) per tensor, so element
    offsets of the last sequences and heads do not fit 32 bits. Inputs are drawn on the GPU from a
    seeded generator (the host copy of a tensor this size would dominate the test); the last
    (sequence, head) unit is checked against the oracle on sampled query rows (O, L, dQ) and
    sampled key columns (dK, dV), whose row statistics the oracle computes blockwise for the whole
    head; the first unit on sampled rows."""
    from paper_2307_08691_amd import binding
    B, N, H, d, scale = 4, 32768, 128, 128, 128 ** -0.5
    gen = torch.Generator(device="cuda").manual_seed(7001)
    draw = lambda: torch.randn(B, N, H, d, device="cuda", dtype=torch.float32, generator=gen).to(torch.bfloat16)  # noqa: E731
    Q = draw()
    K = draw()
    V = draw()
    dO = draw()
    assert Q.numel() == 2 ** 31
    O, L = binding.fa_fwd(Q, K, V, scale, True)
    dQ, dK, dV = binding.fa_bwd(Q, K, V, O, dO, L, scale, True)
    torch.cuda.synchronize()
    rows = np.asarray([0, 1, 255, 256, 12345, 32766, 32767])
    cols = [0, 127, 128, 20000, 32767]
    f64 = lambda t: t.double().cpu().numpy()  # noqa: E731
    for (b, h, full) in ((B - 1, H - 1, True), (0, 0, False)):
        q, k, v, do = f64(Q[b, :, h]), f64(K[b, :, h]), f64(V[b, :, h]), f64(dO[b, :, h])
        o, lse = orc.rows_forward(q[rows], rows, k, v, scale, True)
        dq = orc.rows_backward_dq(q[rows], rows, k, v, do[rows], scale, True)
        for nm, got, exp in (("O", O[b, rows, h], o), ("LSE", L[b, h, rows], lse), ("dQ", dQ[b, rows, h], dq)):
            err = pu.maxdiff(f64(got), exp)
            assert err <= pu.tolerance(nm, exp), f"unit ({b},{h}) {nm}: {err:.3e}"
        if full:
            Lall, _, Dall = orc.head_statistics_blockwise(q, k, v, do, scale, True, block=1024)
            gk, gv = orc.cols_backward_dkdv(q, k[cols], v[cols], cols, N, do, Lall, Dall, scale, True)
            for nm, got, exp in (("dK", dK[b, cols, h], gk), ("dV", dV[b, cols, h], gv)):
                err = pu.maxdiff(f64(got), exp)
                assert err <= pu.tolerance(nm, exp), f"unit ({b},{h}) {nm}: {err:.3e}"
    for t in (O, L, dQ, dK, dV):
        # finiteness of everything, in slices (a 4 GiB tensor widened at once would double the footprint)
        for b in range(B):
            assert torch.isfinite(t[b].float()).all()
