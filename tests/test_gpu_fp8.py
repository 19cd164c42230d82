"""GPU parity for the forward pass on FP8 (E4M3) operands, fa_fp8_fwd, against the float64 oracle run
on the dequantised inputs. Bounds, derived from the arithmetic (the one new error source is the
E4M3 rounding of the probabilities as operands of the second product: 2^-4 relative per entry, and
entries below 2^-17 of a row's maximum flushed to zero):
    |dO| <= (2^-4 + Nk 2^-17) max|V| + half a bf16 ulp of the output,   |dLSE| <= 1e-3,
and the error is no worse than that of an implementation of the same convention that materialises
S and the E4M3 probabilities (torch), plus one bf16 ulp."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402


def fp8_reference_head(q8, k8, v8, dq, dk, dv, scale, causal):
    """Same convention, S and P materialised: torch on the GPU, one head. q8 [Nq,d], k8, v8 [Nk,d] uint8."""
    q, k, v = (t.view(torch.float8_e4m3fn).float() for t in (q8, k8, v8))
    s = (q @ k.T) * (scale * dq * dk)
    if causal:
        n, nk = s.shape
        s = s.masked_fill(torch.ones(n, nk, dtype=torch.bool, device=s.device).triu(1 + nk - n), float("-inf"))
    m = s.max(dim=1, keepdim=True).values
    e = torch.exp(s - m)
    p8 = (e * 256.0).to(torch.float8_e4m3fn).float()
    o = (p8 @ v) * (dv / 256.0) / e.sum(dim=1, keepdim=True)
    return pu.to_f64(o.to(torch.bfloat16)), pu.to_f64(m[:, 0] + torch.log(e.sum(dim=1)))


def judge_fp8(label, O, L, eO, eL, rO, vmax, nk):
    g = pu.to_f64(O)
    assert np.all(np.isfinite(g)) and bool(torch.isfinite(L).all()), label
    err, ref_err = pu.maxdiff(g, eO), pu.maxdiff(rO, eO)
    u = pu.bf16_ulp(pu.maxabs(eO))
    bound = (2.0 ** -4 + nk * 2.0 ** -17) * vmax + 0.5 * u
    lerr = pu.maxdiff(pu.to_f64(L), eL)
    print(f"{label:60s} O err {err:.3e} (bound {bound:.3e}, reference {ref_err:.3e}, ulp {u:.3e})  LSE err {lerr:.3e}")
    assert err <= bound, f"{label}: O err {err:.3e} > {bound:.3e}"
    assert err <= ref_err + u, f"{label}: O err {err:.3e} worse than the materialising FP8 reference {ref_err:.3e} + ulp {u:.3e}"
    assert lerr <= pu.TOL_LSE, f"{label}: LSE err {lerr:.3e}"


def run_fp8(prob):
    dq, dk, dv = prob.meta["descale"]
    Q8, K8, V8 = (torch.from_numpy(x).cuda() for x in (prob.Q, prob.K, prob.V))
    Vt8 = binding.fp8_key_major(V8)
    O, L = binding.fa_fp8_fwd(Q8, K8, Vt8, prob.keys, prob.scale, dq, dk, dv, prob.causal)
    torch.cuda.synchronize()
    return Q8, K8, V8, O, L


def check_fp8(prob):
    dq, dk, dv = prob.meta["descale"]
    Q8, K8, V8, O, L = run_fp8(prob)
    eO, eL = orc.attention_forward_fp8(prob.Q, prob.K, prob.V, dq, dk, dv, prob.scale, prob.causal)
    G = prob.Hq // prob.Hkv
    rO = np.zeros_like(eO)
    for b in range(prob.B):
        for h in range(prob.Hq):
            rO[b, :, h], _ = fp8_reference_head(Q8[b, :, h], K8[b, :, h // G], V8[b, :, h // G], dq, dk, dv, prob.scale, prob.causal)
    vmax = dv * 448.0
    judge_fp8(f"fp8 {pu.describe(prob)}", O, L, eO, eL, rO, vmax, prob.keys)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("N", [1, 2, 31, 63, 64, 65, 128, 257, 300, 515, 1100])
def test_self_attention_on_fp8_operands(N, d, causal):
    check_fp8(inputs.make_fp8(B=2, Nq=N, Nk=N, Hq=2, Hkv=2, d=d, causal=causal, seed=19000 + N + d))


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d", [(1, 300, 8, 2, 128), (70, 333, 4, 2, 64), (257, 1000, 4, 1, 128), (300, 129, 2, 2, 128)])
def test_two_lengths_and_grouped_heads(Nq, Nk, Hq, Hkv, d, causal):
    if causal and Nq > Nk:
        pytest.skip("causal needs at least as many keys as queries")
    check_fp8(inputs.make_fp8(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=19100 + Nq))


def test_exact_cases():
    """One key: P = 1 = 2^8 / 2^8 exactly, so O is that key's dequantised value row rounded to bf16,
    bit for bit, and L its score."""
    prob = inputs.make_fp8(B=1, Nq=5, Nk=1, Hq=2, Hkv=2, d=64, causal=False, seed=19200)
    dq, dk, dv = prob.meta["descale"]
    _, _, _, O, L = run_fp8(prob)
    v = dv * orc.widen_e4m3(prob.V)[0, 0]            # [Hkv, d]
    want = torch.from_numpy(v).to(torch.bfloat16).double().numpy()
    for r in range(5):
        assert np.array_equal(pu.to_f64(O[0, r]), want)
    s = prob.scale * dq * dk * np.einsum("rhd,hd->hr", orc.widen_e4m3(prob.Q)[0], orc.widen_e4m3(prob.K)[0, 0])
    assert pu.maxdiff(pu.to_f64(L[0]), s) <= pu.TOL_LSE


def test_bad_arguments_are_rejected():
    q = torch.zeros(1, 64, 2, 64, dtype=torch.uint8, device="cuda")
    vt = torch.zeros(1, 2, 64, 64, dtype=torch.uint8, device="cuda")
    o = torch.empty(1, 64, 2, 64, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(1, 2, 64, dtype=torch.float32, device="cuda")

    def run(stride=64, d=64, dq=1.0, Nk=64):
        return binding.fa_fp8_fwd_raw(q.data_ptr(), q.data_ptr(), vt.data_ptr(), o.data_ptr(), lse.data_ptr(), 1, 2, 2, 64, Nk, d,
                                      stride, 0.125, dq, 1.0, 1.0, 0, 0)
    assert run() == binding.FA_OK
    assert run(stride=32) == binding.FA_ERR_SHAPE
    assert run(stride=96) == binding.FA_ERR_SHAPE
    assert run(d=32) == binding.FA_ERR_UNSUPPORTED
    assert run(dq=0.0) == binding.FA_ERR_SHAPE
    assert run(dq=float("inf")) == binding.FA_ERR_SHAPE
    torch.cuda.synchronize()


def test_full_size_fp8_workload_sampled_units():
    """The benchmark shape (B=2, N=8192, 16 heads of 128, causal) on E4M3 operands; two whole units."""
    prob = inputs.make_fp8(B=2, Nq=8192, Nk=8192, Hq=16, Hkv=16, d=128, causal=True, seed=19300)
    dq, dk, dv = prob.meta["descale"]
    Q8, K8, V8, O, L = run_fp8(prob)
    assert torch.isfinite(O.float()).all() and torch.isfinite(L).all()
    for (b, h) in ((0, 0), (1, 15)):
        q, k, v = dq * orc.widen_e4m3(prob.Q[b, :, h]), dk * orc.widen_e4m3(prob.K[b, :, h]), dv * orc.widen_e4m3(prob.V[b, :, h])
        o, lse, _ = orc.head_forward(q, k, v, prob.scale, True)
        ro, _ = fp8_reference_head(Q8[b, :, h], K8[b, :, h], V8[b, :, h], dq, dk, dv, prob.scale, True)
        judge_fp8(f"fp8 d128 N8192 causal unit ({b},{h})", O[b, :, h], L[b, h], o, lse, ro, dv * 448.0, 8192)
