"""GPU parity for head dimensions other than the two tile widths: any multiple of 8 up to 128
goes through the same entry points, the kernels padding rows with zeros on chip. Checked element
by element against the float64 oracle (which has no notion of padding), with guard values around
every output so that a store past a row's real length would show."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402
from test_gpu_parity import check  # noqa: E402
from test_gpu_cross import ragged_cross  # noqa: E402


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [8, 32, 40, 56, 72, 96, 120])
@pytest.mark.parametrize("N", [1, 65, 300, 515])
def test_self_attention_at_other_head_dimensions(N, d, causal):
    prob = inputs.make_dense(B=2, N=N, Hq=2, Hkv=2, d=d, causal=causal, seed=8000 + N + d)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d,dtype", [(70, 333, 4, 2, 96, "bf16"), (1, 300, 8, 2, 32, "bf16"),
                                                  (300, 301, 4, 1, 80, "f16"), (129, 257, 2, 2, 32, "f16")])
def test_two_lengths_grouped_heads_and_half_precision(Nq, Nk, Hq, Hkv, d, dtype, causal):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=8100 + d, dtype=dtype)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [32, 96])
def test_packed_ragged_batches(d, causal):
    prob = inputs.make_varlen([100, 257, 1, 31, 300], Hq=4, Hkv=2, d=d, causal=causal, seed=8200 + d)
    check(prob)


@pytest.mark.parametrize("d", [32, 96])
def test_packed_ragged_batches_with_two_lengths(d):
    lq, lk = [1, 70, 0, 300], [257, 70, 33, 515]
    cu_q, cu_k, Qb, Kb, Vb, dOb = ragged_cross(lq, lk, 4, 2, d, 8300 + d)
    Q, K, V, dO = (pu.to_gpu(x) for x in (Qb, Kb, Vb, dOb))
    cq, ck = torch.from_numpy(cu_q).cuda(), torch.from_numpy(cu_k).cuda()
    scale = d ** -0.5
    O, L = binding.fa_varlen_cross_fwd(Q, K, V, cq, ck, max(lq), max(lk), scale, True)
    dQ, dK, dV = binding.fa_varlen_cross_bwd(Q, K, V, O, dO, L, cq, ck, max(lq), max(lk), scale, True)
    torch.cuda.synchronize()
    Qf, Kf, Vf, dOf = (orc.widen_bf16(x) for x in (Qb, Kb, Vb, dOb))
    eO, eL = orc.varlen_forward(Qf, Kf, Vf, cu_q, scale, True, cu_seqlens_k=cu_k)
    edQ, edK, edV = orc.varlen_backward(Qf, Kf, Vf, dOf, cu_q, scale, True, cu_seqlens_k=cu_k)
    ref = pu.reference_batch(Q, K, V, dO, scale, True, cu_q=cu_q, cu_k=cu_k)
    pu.judge(f"ragged, two lengths, d{d}", {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))},
             dict(O=eO, LSE=eL, dQ=edQ, dK=edK, dV=edV), ref, d=d)


@pytest.mark.parametrize("d", [24, 96])
def test_nothing_is_written_past_a_rows_real_length(d):
    """Outputs live inside larger buffers filled with a guard pattern: rows are d elements long in
    memory although the kernels work on 64- or 128-wide tiles."""
    prob = inputs.make_dense(B=1, N=130, Hq=2, Hkv=2, d=d, causal=True, seed=8400 + d)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    pad = 4096

    def guarded(like):
        buf = torch.full((like.numel() + 2 * pad,), 7.0, dtype=torch.bfloat16, device="cuda")
        return buf, buf[pad:pad + like.numel()].view(like.shape)

    bO, O = guarded(Q)
    bQ, dQ = guarded(Q)
    bK, dK = guarded(K)
    bV, dV = guarded(V)
    O, L = binding.fa_fwd(Q, K, V, prob.scale, True, O=O)
    binding.fa_bwd(Q, K, V, O, dO, L, prob.scale, True, dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    for buf in (bO, bQ, bK, bV):
        assert bool((buf[:pad] == 7.0).all()) and bool((buf[-pad:] == 7.0).all())
    pu.judge(f"guarded outputs, d{d}", {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))},
             pu.run_oracle(prob), pu.run_reference(prob), d=d)


def test_dropout_and_split_keys_keep_to_the_tile_widths():
    q = torch.zeros(1, 8, 2, 96, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(RuntimeError):
        binding.fa_dropout_fwd(q, q, q, 0.1, False, 0.1, 1)
    with pytest.raises(RuntimeError):
        binding.fa_splitkv_fwd(q, q, q, 0.1, False, num_splits=2)
    k = torch.zeros(1, 8, 2, 136, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(RuntimeError):
        binding.fa_fwd(k, k, k, 0.1, False)
