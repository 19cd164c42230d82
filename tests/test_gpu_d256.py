"""GPU parity at head dimension 256 (kernels of their own: four wavefronts with 512 registers
each, fa_d256.hip): forward and backward against the float64 oracle through the dense, packed
ragged, two-length and half precision entry points, at sizes that span several 128-row blocks,
ragged tails, grouped heads and the causal alignment of two lengths."""
import pytest

from paper_2307_08691_amd import binding, inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402
from test_gpu_parity import check  # noqa: E402
from test_gpu_fullsize import check_units  # noqa: E402


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N", [1, 31, 64, 128, 129, 300, 517, 1000])
def test_self_attention(N, causal):
    prob = inputs.make_dense(B=2, N=N, Hq=2, Hkv=2, d=256, causal=causal, seed=18000 + N)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (8, 1), (6, 3)])
def test_grouped_heads(Hq, Hkv, causal):
    prob = inputs.make_dense(B=2, N=333, Hq=Hq, Hkv=Hkv, d=256, causal=causal, seed=18100 + Hq)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
def test_packed_ragged_batch(causal):
    prob = inputs.make_varlen([5, 130, 0, 64, 257, 1, 300, 128], Hq=4, Hkv=2, d=256, causal=causal, seed=18200)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Nq,Nk", [(1, 300), (70, 333), (200, 1000), (257, 300)])
def test_two_lengths(Nq, Nk, causal):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=4, Hkv=2, d=256, causal=causal, seed=18300 + Nq)
    check(prob)


def test_more_queries_than_keys_without_mask():
    prob = inputs.make_cross(B=2, Nq=300, Nk=129, Hq=2, Hkv=2, d=256, causal=False, seed=18400)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
def test_half_precision(causal):
    prob = inputs.make_cross(B=2, Nq=300, Nk=300, Hq=4, Hkv=2, d=256, causal=causal, seed=18500, dtype="f16")
    check(prob)


def test_wide_score_range():
    prob = inputs.make_dense(B=1, N=700, Hq=2, Hkv=1, d=256, causal=True, seed=18600, qk_mult=3.0)
    check(prob)


def test_full_size_sampled_units():
    """16k tokens in 8 heads of 256 (the paper's hidden dimension 2048), N = 4096, causal."""
    prob = inputs.make_dense(B=4, N=4096, Hq=8, Hkv=8, d=256, causal=True, seed=18700)
    got = pu.run_hip(prob)
    for nm, t in got.items():
        assert torch.isfinite(t.float()).all(), nm
    print(check_units(prob, got, [(0, 0), (3, 7)]))


def test_options_stay_at_the_two_tile_widths():
    q = torch.zeros(1, 8, 2, 256, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.FaError) as e:
        binding.fa_dropout_fwd(q, q, q, 0.1, True, 0.1, 7)
    assert e.value.status == binding.FA_ERR_UNSUPPORTED
