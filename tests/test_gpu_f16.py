"""GPU parity for IEEE half precision elements (fa_cross_fwd_f16 / fa_cross_bwd_f16): the same
cases as for bfloat16, on inputs rounded to fp16, against the float64 oracle run on exactly those
fp16 values. fp16 carries three more significand bits than bfloat16, so the bfloat16 bounds hold
with room; the yardstick implementation materialising S and P is run in fp16 as well."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402
from test_gpu_parity import check  # noqa: E402
from test_gpu_fullsize import check_units  # noqa: E402


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
