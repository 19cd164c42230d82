"""GPU parity for IEEE half precision elements (fa_cross_fwd_f16 / fa_cross_bwd_f16): the same
cases as for bfloat16, on inputs rounded to fp16, against the float64 oracle run on exactly those
fp16 values. fp16 carries three more significand bits than bfloat16, so the bfloat16 bounds hold
with room; the yardstick implementation materialising S and P is run in fp16 as well."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402
from test_gpu_parity import check  # noqa: E402
from test_gpu_fullsize import check_units  # noqa: E402
from test_gpu_kvcache import reference as cache_reference  # noqa: E402


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("N", [1, 63, 65, 128, 257, 515])
def test_self_attention_in_half_precision(N, d, causal):
    prob = inputs.make_cross(B=2, Nq=N, Nk=N, Hq=2, Hkv=2, d=d, causal=causal, seed=5000 + N, dtype="f16")
    errs = check(prob)
    # three more significand bits than bfloat16 show: well inside the bfloat16 bounds
    assert errs["O"] <= 5e-3 and errs["LSE"] <= 1e-3


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d", [(1, 300, 8, 2, 128), (70, 333, 4, 2, 64), (300, 129, 2, 2, 128)])
def test_two_lengths_and_grouped_heads_in_half_precision(Nq, Nk, Hq, Hkv, d, causal):
    if causal and Nq > Nk:
        pytest.skip("causal needs at least as many keys as queries")
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=5100 + Nq, dtype="f16")
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d,Hq,Hkv", [(64, 2, 2), (128, 4, 2), (96, 2, 1)])
def test_ragged_batches_in_half_precision(d, Hq, Hkv, causal):
    check(inputs.make_varlen([100, 257, 1, 0, 31, 515], Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=5300 + d, dtype="f16"))


@pytest.mark.parametrize("causal", [False, True])
def test_ragged_batches_with_two_lengths_in_half_precision(causal):
    """fa_varlen_cross_fwd_f16 / bwd_f16, including a sequence without queries and one without keys."""
    lq, lk = [10, 70, 0, 1, 200, 5], [100, 333, 50, 300, 257, 0 if not causal else 5]
    Hq, Hkv, d = 4, 2, 128
    g = np.random.default_rng(5400)
    cu_q, cu_k = (np.concatenate([[0], np.cumsum(x)]).astype(np.int32) for x in (lq, lk))
    bits = lambda shape: inputs.f32_to_f16_bits(g.standard_normal(shape, dtype=np.float32))  # noqa: E731
    Qb, dOb = bits((cu_q[-1], Hq, d)), bits((cu_q[-1], Hq, d))
    Kb, Vb = bits((cu_k[-1], Hkv, d)), bits((cu_k[-1], Hkv, d))
    Q, K, V, dO = (pu.to_gpu(x, "f16") for x in (Qb, Kb, Vb, dOb))
    cq, ck = torch.from_numpy(cu_q).cuda(), torch.from_numpy(cu_k).cuda()
    scale = d ** -0.5
    O, L = binding.fa_varlen_cross_fwd(Q, K, V, cq, ck, max(lq), max(lk), scale, causal)
    dQ, dK, dV = binding.fa_varlen_cross_bwd(Q, K, V, O, dO, L, cq, ck, max(lq), max(lk), scale, causal)
    torch.cuda.synchronize()
    assert O.dtype == torch.float16 and dK.dtype == torch.float16
    Qf, Kf, Vf, dOf = (orc.widen_f16(x) for x in (Qb, Kb, Vb, dOb))
    exp = {}
    exp["O"], exp["LSE"] = orc.varlen_forward(Qf, Kf, Vf, cu_q, scale, causal, cu_k)
    exp["dQ"], exp["dK"], exp["dV"] = orc.varlen_backward(Qf, Kf, Vf, dOf, cu_q, scale, causal, cu_k)
    ref = pu.reference_batch(Q, K, V, dO, scale, causal, cu_q=cu_q, cu_k=cu_k)
    pu.judge(f"ragged two lengths f16 causal={causal}",
             {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))}, exp, ref,
             dtype="f16", d=d)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d,splits", [(1, 1000, 8, 2, 128, 3), (5, 700, 4, 4, 64, 2), (70, 4097, 8, 1, 128, 0)])
def test_split_keys_and_the_key_value_cache_in_half_precision(Nq, Nk, Hq, Hkv, d, splits, causal):
    prob = inputs.make_cross(B=3, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=5500 + Nq, dtype="f16")
    Q, K, V = (pu.to_gpu(x, "f16") for x in (prob.Q, prob.K, prob.V))
    O, L = binding.fa_splitkv_fwd(Q, K, V, prob.scale, causal, splits)
    lens = [Nk, max(Nq, 1), Nk // 2 + 3]
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    O2, L2 = binding.fa_kvcache_fwd(Q, K, V, prob.scale, causal, seqlens_k=sl, num_splits=splits)
    torch.cuda.synchronize()
    assert O.dtype == torch.float16 and O2.dtype == torch.float16
    Qf, Kf, Vf = (orc.widen_f16(x) for x in (prob.Q, prob.K, prob.V))
    eO, eL = orc.attention_forward(Qf, Kf, Vf, prob.scale, causal)
    ref = pu.reference_batch(Q, K, V, torch.zeros_like(Q), prob.scale, causal, backward=False)
    pu.judge(f"split keys f16 {pu.describe(prob)}", {"O": pu.to_f64(O), "LSE": pu.to_f64(L)}, {"O": eO, "LSE": eL}, ref,
             dtype="f16", d=d)
    eO2, eL2 = orc.kvcache_forward(Qf, Kf, Vf, prob.scale, causal, np.asarray(lens))
    ref2 = cache_reference(Q, lambda b: K[b, :lens[b]], lambda b: V[b, :lens[b]], lens, prob.scale, causal, Hq, Hkv)
    pu.judge(f"cache f16 {lens} {pu.describe(prob)}", {"O": pu.to_f64(O2), "LSE": pu.to_f64(L2)}, {"O": eO2, "LSE": eL2}, ref2,
             dtype="f16", d=d)


def test_half_precision_outputs_are_half_precision_roundings():
    """The stored O is the fp16 rounding of a value close to the exact one: half an fp16 ulp plus
    the arithmetic error, far below a bfloat16 ulp."""
    prob = inputs.make_cross(B=1, Nq=200, Nk=200, Hq=2, Hkv=2, d=64, causal=False, seed=5200, dtype="f16")
    got = pu.run_hip(prob, backward=False)
    exp = pu.run_oracle(prob, backward=False)
    assert got["O"].dtype == torch.float16
    assert pu.maxdiff(pu.to_f64(got["O"]), exp["O"]) <= 2e-3


def test_mixed_element_types_are_rejected_by_the_binding():
    q = torch.zeros(1, 8, 2, 64, dtype=torch.float16, device="cuda")
    k = torch.zeros(1, 8, 2, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):
        binding.fa_cross_fwd(q, k, k, 0.125, False)


def test_full_size_half_precision_workload_sampled_units():
    prob = inputs.make_config("f16_d128_n8k_causal")
    got = pu.run_hip(prob)
    for nm, t in got.items():
        assert torch.isfinite(t.float()).all(), nm
    print(prob.name, check_units(prob, got, [(0, 0), (1, 15)]))
