"""GPU parity for two lengths (Nq query rows against Nk key/value rows): the HIP path
through fa_cross_fwd / fa_cross_bwd against the float64 oracle, element by element, at
sizes that span several tiles, ragged tails on either side, a single query row, more
queries than keys (no mask), grouped heads; plus the identity with the one-length entry
points and sampled units of the two full-size workloads."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402
from test_gpu_parity import check  # noqa: E402
from test_gpu_fullsize import check_units  # noqa: E402


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Nq,Nk", [(1, 1), (1, 300), (7, 64), (31, 129), (64, 65), (128, 515), (200, 1000),
                                   (257, 300), (300, 301), (33, 2049)])
def test_fewer_queries_than_keys(Nq, Nk, d, causal):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=2, Hkv=2, d=d, causal=causal, seed=3000 + Nq + Nk)
    check(prob)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Nq,Nk", [(64, 7), (300, 129), (515, 64), (129, 1)])
def test_more_queries_than_keys_without_mask(Nq, Nk, d):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=2, Hkv=2, d=d, causal=False, seed=3100 + Nq + Nk)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d,Hq,Hkv", [(64, 4, 2), (128, 8, 2), (128, 4, 1)])
def test_grouped_heads_with_two_lengths(d, Hq, Hkv, causal):
    prob = inputs.make_cross(B=2, Nq=70, Nk=333, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=3200 + Hq)
    check(prob)


def test_single_new_token_against_a_cache():
    """Decoding shape: one query row per sequence, grouped heads, a long key sequence."""
    prob = inputs.make_cross(B=4, Nq=1, Nk=4097, Hq=8, Hkv=2, d=128, causal=True, seed=3300)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
def test_equal_lengths_reproduce_the_one_length_entry_points_bitwise(causal):
    prob = inputs.make_dense(B=2, N=300, Hq=4, Hkv=2, d=128, causal=causal, seed=3400)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    O1, L1 = binding.fa_fwd(Q, K, V, prob.scale, causal)
    O2, L2 = binding.fa_cross_fwd(Q, K, V, prob.scale, causal)
    g1 = binding.fa_bwd(Q, K, V, O1, dO, L1, prob.scale, causal)
    g2 = binding.fa_cross_bwd(Q, K, V, O2, dO, L2, prob.scale, causal)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(L1, L2)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


def test_causal_chunk_equals_the_last_rows_of_the_square_problem():
    """The newest Nq rows of a causal self-attention problem, run through the two-length
    entry points, give the same O and LSE rows (same keys, same alignment)."""
    prob = inputs.make_dense(B=1, N=777, Hq=2, Hkv=2, d=64, causal=True, seed=3500)
    Q, K, V = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V))
    O, L = binding.fa_fwd(Q, K, V, prob.scale, True)
    nq = 200
    Oc, Lc = binding.fa_cross_fwd(Q[:, -nq:].contiguous(), K, V, prob.scale, True)
    torch.cuda.synchronize()
    assert float((O[:, -nq:].float() - Oc.float()).abs().max()) <= 2e-2
    assert float((L[:, :, -nq:] - Lc).abs().max()) <= 1e-3


def test_guard_values_around_outputs_survive():
    """Outputs of different lengths: nothing is written outside dQ (Nq rows) or dK, dV (Nk rows)."""
    prob = inputs.make_cross(B=1, Nq=37, Nk=211, Hq=2, Hkv=2, d=64, causal=True, seed=3600)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    pad = 4096

    def guarded(like):
        buf = torch.full((like.numel() + 2 * pad,), 7.0, dtype=torch.bfloat16, device="cuda")
        return buf, buf[pad:pad + like.numel()].view(like.shape)

    bO, O = guarded(Q)
    bQ, dQ = guarded(Q)
    bK, dK = guarded(K)
    bV, dV = guarded(V)
    O, L = binding.fa_cross_fwd(Q, K, V, prob.scale, True, O=O)
    binding.fa_cross_bwd(Q, K, V, O, dO, L, prob.scale, True, dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    for buf in (bO, bQ, bK, bV):
        assert bool((buf[:pad] == 7.0).all()) and bool((buf[-pad:] == 7.0).all())
    pu.judge("guarded outputs, two lengths", {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))},
             pu.run_oracle(prob), pu.run_reference(prob), d=prob.d)


@pytest.mark.parametrize("name", ["chunk_512_on_8k", "cross_2k_on_8k"])
def test_full_size_two_length_workloads_sampled_units(name):
    prob = inputs.make_config(name)
    got = pu.run_hip(prob)
    for nm, t in got.items():
        assert torch.isfinite(t.float()).all(), f"{name}: {nm} not finite"
    units = [(0, 0), (prob.B - 1, prob.Hkv - 1)]
    worst = check_units(prob, got, units)
    print(name, worst)


# ---------------------------------------------------------------------------------------------
# key sequence split over workgroups (fa_splitkv_fwd): same result as the definition
# ---------------------------------------------------------------------------------------------

def check_splitkv(prob, num_splits):
    Q, K, V = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V))
    O, L = binding.fa_splitkv_fwd(Q, K, V, prob.scale, prob.causal, num_splits)
    torch.cuda.synchronize()
    pu.judge(f"split keys {pu.describe(prob)} shares={num_splits}", {"O": pu.to_f64(O), "LSE": pu.to_f64(L)},
             pu.run_oracle(prob, backward=False), pu.run_reference(prob, backward=False), d=prob.d)
    return O, L


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("num_splits", [1, 2, 3, 7, 0])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d", [(1, 1, 2, 2, 64), (1, 300, 8, 2, 128), (1, 4097, 8, 1, 128), (3, 65, 4, 4, 64),
                                            (17, 1000, 6, 2, 128), (100, 129, 4, 2, 64), (70, 515, 8, 2, 128)])
def test_split_keys_match_the_oracle(Nq, Nk, Hq, Hkv, d, num_splits, causal):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=3700 + Nq + Nk)
    check_splitkv(prob, num_splits)


def test_more_shares_than_key_blocks_and_rows_without_keys_in_a_share():
    """Causal, the first queries see only the first keys: most shares hold nothing for them."""
    prob = inputs.make_cross(B=1, Nq=200, Nk=260, Hq=2, Hkv=1, d=64, causal=True, seed=3800)
    check_splitkv(prob, 5)    # 5 blocks of 64 keys, one per share
    check_splitkv(prob, 40)   # 35 empty shares


def test_split_keys_agree_with_the_unsplit_entry_point():
    prob = inputs.make_cross(B=3, Nq=5, Nk=2049, Hq=8, Hkv=2, d=128, causal=True, seed=3900)
    Q, K, V = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V))
    O1, L1 = binding.fa_cross_fwd(Q, K, V, prob.scale, True)
    O2, L2 = check_splitkv(prob, 6)
    assert float((O1.float() - O2.float()).abs().max()) <= 2 * pu.bf16_ulp(float(O1.float().abs().max()))
    assert float((L1 - L2).abs().max()) <= 1e-4


# ---------------------------------------------------------------------------------------------
# packed ragged batches with two lengths per sequence
# ---------------------------------------------------------------------------------------------

def ragged_cross(lq, lk, Hq, Hkv, d, seed):
    rng = np.random.default_rng(seed)
    cu_q = np.concatenate([[0], np.cumsum(lq)]).astype(np.int32)
    cu_k = np.concatenate([[0], np.cumsum(lk)]).astype(np.int32)
    draw = lambda *shape: inputs.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))
    return cu_q, cu_k, draw(cu_q[-1], Hq, d), draw(cu_k[-1], Hkv, d), draw(cu_k[-1], Hkv, d), draw(cu_q[-1], Hq, d)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d,Hq,Hkv", [(64, 2, 2), (128, 8, 2)])
def test_ragged_batches_with_two_lengths(d, Hq, Hkv, causal):
    lq = [1, 70, 0, 300, 64, 5]
    lk = [257, 70, 33, 515, 65, 1000]
    cu_q, cu_k, Qb, Kb, Vb, dOb = ragged_cross(lq, lk, Hq, Hkv, d, 4000 + d)
    Q, K, V, dO = (pu.to_gpu(x) for x in (Qb, Kb, Vb, dOb))
    cq, ck = torch.from_numpy(cu_q).cuda(), torch.from_numpy(cu_k).cuda()
    scale = d ** -0.5
    O, L = binding.fa_varlen_cross_fwd(Q, K, V, cq, ck, max(lq), max(lk), scale, causal)
    dQ, dK, dV = binding.fa_varlen_cross_bwd(Q, K, V, O, dO, L, cq, ck, max(lq), max(lk), scale, causal)
    torch.cuda.synchronize()
    Qf, Kf, Vf, dOf = (orc.widen_bf16(x) for x in (Qb, Kb, Vb, dOb))
    eO, eL = orc.varlen_forward(Qf, Kf, Vf, cu_q, scale, causal, cu_seqlens_k=cu_k)
    edQ, edK, edV = orc.varlen_backward(Qf, Kf, Vf, dOf, cu_q, scale, causal, cu_seqlens_k=cu_k)
    ref = pu.reference_batch(Q, K, V, dO, scale, causal, cu_q=cu_q, cu_k=cu_k)
    pu.judge(f"ragged, two lengths, d{d} H{Hq}/{Hkv} causal={causal}",
             {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))},
             dict(O=eO, LSE=eL, dQ=edQ, dK=edK, dV=edV), ref, d=d)
    # the keys of the sequence without queries receive exactly zero
    assert not bool(dK[cu_k[2]:cu_k[3]].any()) and not bool(dV[cu_k[2]:cu_k[3]].any())


@pytest.mark.parametrize("d", [64, 128, 256, 96])
def test_a_sequence_with_queries_but_no_keys(d):
    """Ragged batch with two lengths, no mask: the first and a middle sequence have no key at all.
    Their rows get O = 0, L = -inf, dQ = 0 (nothing is read before the key/value base), the
    other sequences are unaffected."""
    lq, lk, Hq, Hkv = [300, 70, 5, 64], [0, 257, 0, 65], 4, 2
    cu_q, cu_k, Qb, Kb, Vb, dOb = ragged_cross(lq, lk, Hq, Hkv, d, 4200 + d)
    Q, K, V, dO = (pu.to_gpu(x) for x in (Qb, Kb, Vb, dOb))
    cq, ck = torch.from_numpy(cu_q).cuda(), torch.from_numpy(cu_k).cuda()
    scale = d ** -0.5
    O, L = binding.fa_varlen_cross_fwd(Q, K, V, cq, ck, max(lq), max(lk), scale, False)
    dQ, dK, dV = binding.fa_varlen_cross_bwd(Q, K, V, O, dO, L, cq, ck, max(lq), max(lk), scale, False)
    torch.cuda.synchronize()
    Qf, Kf, Vf, dOf = (orc.widen_bf16(x) for x in (Qb, Kb, Vb, dOb))
    eO, eL = orc.varlen_forward(Qf, Kf, Vf, cu_q, scale, False, cu_seqlens_k=cu_k)
    edQ, edK, edV = orc.varlen_backward(Qf, Kf, Vf, dOf, cu_q, scale, False, cu_seqlens_k=cu_k)
    ref = pu.reference_batch(Q, K, V, dO, scale, False, cu_q=cu_q, cu_k=cu_k)
    ref["LSE"][:, :300] = -np.inf   # (the reference skips sequences it cannot run)
    ref["LSE"][:, 370:375] = -np.inf
    pu.judge(f"ragged with keyless sequences, d{d}", {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))},
             dict(O=eO, LSE=eL, dQ=edQ, dK=edK, dV=edV), ref, d=d)
    for a, e in ((0, 300), (370, 375)):
        assert not bool(O[a:e].any()) and not bool(dQ[a:e].any()) and bool(torch.isneginf(L[:, a:e]).all())


def test_ragged_two_lengths_with_equal_offsets_reproduce_the_one_length_entry_points():
    prob = inputs.make_varlen([100, 257, 31], Hq=4, Hkv=2, d=128, causal=True, seed=4100)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    cu = torch.from_numpy(prob.cu_seqlens.astype(np.int32)).cuda()
    O1, L1 = binding.fa_varlen_fwd(Q, K, V, cu, 257, prob.scale, True)
    O2, L2 = binding.fa_varlen_cross_fwd(Q, K, V, cu, cu.clone(), 257, 257, prob.scale, True)
    g1 = binding.fa_varlen_bwd(Q, K, V, O1, dO, L1, cu, 257, prob.scale, True)
    g2 = binding.fa_varlen_cross_bwd(Q, K, V, O2, dO, L2, cu, cu.clone(), 257, 257, prob.scale, True)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(L1, L2)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)
