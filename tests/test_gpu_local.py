"""GPU parity for local (sliding-window) attention, fa_local_fwd / fa_local_bwd, against the float64
oracle's window pattern: windows narrower and wider than the kernels' tiles (32-row wavefront
slices, 64-key blocks, 256-row and 256-key workgroup blocks), bounds on one side only, two lengths,
grouped heads; the reductions to plain and causal attention; sampled units at full size."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402


def window_mask_gpu(nq, nk, left, right):
    """The window as an additive mask [1, 1, nq, nk] (0 / -inf) for the 16-bit reference."""
    p = torch.arange(nq, device="cuda")[:, None] + (nk - nq)
    c = torch.arange(nk, device="cuda")[None, :]
    vis = torch.ones(nq, nk, dtype=torch.bool, device="cuda")
    if left >= 0:
        vis &= c >= p - left
    if right >= 0:
        vis &= c <= p + right
    return torch.where(vis, 0.0, float("-inf"))[None, None]


def check_local(prob, left, right):
    Q, K, V, dO = (pu.to_gpu(x, prob.dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    O, L = binding.fa_local_fwd(Q, K, V, prob.scale, left, right)
    dQ, dK, dV = binding.fa_local_bwd(Q, K, V, O, dO, L, prob.scale, left, right)
    torch.cuda.synchronize()
    widen = orc.widen_f16 if prob.dtype == "f16" else orc.widen_bf16
    Qf, Kf, Vf, dOf = (widen(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    exp = {}
    exp["O"], exp["LSE"] = orc.attention_forward_local(Qf, Kf, Vf, prob.scale, left, right)
    exp["dQ"], exp["dK"], exp["dV"] = orc.attention_backward_local(Qf, Kf, Vf, dOf, prob.scale, left, right)
    ref = pu.reference_batch(Q, K, V, dO, prob.scale, False, M=window_mask_gpu(prob.N, prob.keys, left, right))
    pu.judge(f"window ({left},{right}) {pu.describe(prob)}",
             {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))}, exp, ref,
             dtype=prob.dtype, d=prob.d)
    return O, L, dQ, dK, dV


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Nq,Nk,left,right", [(65, 65, 3, 3), (300, 1000, 128, 0), (700, 700, 31, 0), (700, 700, 200, 5),
                                             (515, 515, -1, 40), (515, 515, 256, 256)])
def test_windows_in_half_precision(Nq, Nk, left, right, d):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=4, Hkv=2, d=d, causal=False, seed=16050 + Nq + Nk + left, dtype="f16")
    check_local(prob, left, right)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("left,right", [(0, 0), (7, 0), (31, 0), (32, 0), (63, 0), (64, 0), (100, 0), (255, 0), (256, 0), (300, 0),
                                        (600, 0), (16, 16), (64, 64), (5, 200), (200, 5), (-1, 40), (40, -1), (0, 33)])
def test_windows_around_every_tile_edge(left, right, d):
    prob = inputs.make_dense(B=2, N=700, Hq=2, Hkv=2, d=d, causal=False, seed=16000 + left + 7 * right)
    check_local(prob, left, right)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Nq,Nk,left,right", [(1, 1, 0, 0), (1, 300, 10, 0), (65, 65, 3, 3), (70, 333, 100, 0), (257, 300, 64, 10),
                                             (300, 1000, 128, 0), (515, 515, 256, 256), (129, 1025, 30, 30)])
def test_two_lengths_and_ragged_tails(Nq, Nk, left, right, d):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=2, Hkv=2, d=d, causal=False, seed=16100 + Nq + Nk)
    check_local(prob, left, right)


@pytest.mark.parametrize("d,Hq,Hkv", [(64, 4, 2), (128, 8, 2), (128, 4, 1)])
def test_grouped_heads(d, Hq, Hkv):
    prob = inputs.make_cross(B=2, Nq=400, Nk=520, Hq=Hq, Hkv=Hkv, d=d, causal=False, seed=16200 + Hq)
    check_local(prob, 90, 0)
    check_local(prob, 40, 70)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("d,Hq,Hkv", [(64, 2, 2), (128, 4, 2)])
@pytest.mark.parametrize("left,right", [(0, 0), (31, 0), (100, 0), (300, 0), (40, 70), (-1, 40), (64, -1)])
def test_windows_inside_the_sequences_of_a_ragged_batch(left, right, d, Hq, Hkv, dtype):
    """fa_varlen_local_fwd / bwd: sequences shorter and longer than the window and than the kernels'
    blocks, one of one token, one without tokens; positions count from each sequence's start."""
    lens = [100, 257, 1, 0, 31, 700, 64]
    prob = inputs.make_varlen(lens, Hq=Hq, Hkv=Hkv, d=d, causal=False, seed=16600 + d + left, dtype=dtype)
    Q, K, V, dO = (pu.to_gpu(x, dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    cu = torch.from_numpy(prob.cu_seqlens.astype(np.int32)).cuda()
    O, L = binding.fa_varlen_local_fwd(Q, K, V, cu, max(lens), prob.scale, left, right)
    dQ, dK, dV = binding.fa_varlen_local_bwd(Q, K, V, O, dO, L, cu, max(lens), prob.scale, left, right)
    torch.cuda.synchronize()
    widen = orc.widen_f16 if dtype == "f16" else orc.widen_bf16
    Qf, Kf, Vf, dOf = (widen(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    exp = {}
    exp["O"], exp["LSE"] = orc.varlen_forward_local(Qf, Kf, Vf, prob.cu_seqlens, prob.scale, left, right)
    exp["dQ"], exp["dK"], exp["dV"] = orc.varlen_backward_local(Qf, Kf, Vf, dOf, prob.cu_seqlens, prob.scale, left, right)
    ref = pu.reference_batch(Q, K, V, dO, prob.scale, False, cu_q=prob.cu_seqlens,
                             M_of=lambda s, h, nq, nk: window_mask_gpu(nq, nk, left, right)[0, 0])
    pu.judge(f"ragged window ({left},{right}) d{d} H{Hq}/{Hkv}",
             {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))}, exp, ref,
             dtype=dtype, d=d)


def test_ragged_bounds_that_bind_nothing_are_the_ragged_entry_points_bitwise():
    prob = inputs.make_varlen([100, 257, 31, 300], Hq=4, Hkv=2, d=128, causal=False, seed=16700)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    cu = torch.from_numpy(prob.cu_seqlens.astype(np.int32)).cuda()
    for (left, right, causal) in ((-1, -1, False), (300, 400, False), (-1, 0, True), (1000, 0, True)):
        O1, L1 = binding.fa_varlen_local_fwd(Q, K, V, cu, 300, prob.scale, left, right)
        O2, L2 = binding.fa_varlen_fwd(Q, K, V, cu, 300, prob.scale, causal)
        g1 = binding.fa_varlen_local_bwd(Q, K, V, O1, dO, L1, cu, 300, prob.scale, left, right)
        g2 = binding.fa_varlen_bwd(Q, K, V, O2, dO, L2, cu, 300, prob.scale, causal)
        torch.cuda.synchronize()
        assert torch.equal(O1, O2) and torch.equal(L1, L2)
        for a, b in zip(g1, g2):
            assert torch.equal(a, b)


def test_bounds_that_bind_nothing_are_plain_and_causal_attention_bitwise():
    prob = inputs.make_cross(B=2, Nq=300, Nk=420, Hq=4, Hkv=2, d=128, causal=False, seed=16300)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    for (left, right, causal) in ((-1, -1, False), (420, 500, False), (-1, 0, True), (1000, 0, True)):
        O1, L1 = binding.fa_local_fwd(Q, K, V, prob.scale, left, right)
        O2, L2 = binding.fa_cross_fwd(Q, K, V, prob.scale, causal)
        g1 = binding.fa_local_bwd(Q, K, V, O1, dO, L1, prob.scale, left, right)
        g2 = binding.fa_cross_bwd(Q, K, V, O2, dO, L2, prob.scale, causal)
        torch.cuda.synchronize()
        assert torch.equal(O1, O2) and torch.equal(L1, L2)
        for a, b in zip(g1, g2):
            assert torch.equal(a, b)


def test_a_window_as_wide_as_the_causal_triangle_matches_the_causal_kernel():
    """left = Nk - 1 binds nothing either, but is below the cut-off that routes to the causal kernel:
    the window kernels must then reproduce causal attention (to rounding: other instantiation)."""
    prob = inputs.make_dense(B=1, N=520, Hq=2, Hkv=2, d=128, causal=True, seed=16400)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    O1, L1 = binding.fa_local_fwd(Q, K, V, prob.scale, 519, 0)
    O2, L2 = binding.fa_fwd(Q, K, V, prob.scale, True)
    g1 = binding.fa_local_bwd(Q, K, V, O1, dO, L1, prob.scale, 519, 0)
    g2 = binding.fa_bwd(Q, K, V, O2, dO, L2, prob.scale, True)
    torch.cuda.synchronize()
    assert float((O1.float() - O2.float()).abs().max()) <= 2 * pu.bf16_ulp(float(O2.float().abs().max()))
    assert float((L1 - L2).abs().max()) <= 1e-5
    for a, b in zip(g1, g2):
        assert float((a.float() - b.float()).abs().max()) <= 2 * pu.bf16_ulp(float(b.float().abs().max()))


def test_outputs_stay_inside_their_buffers():
    prob = inputs.make_cross(B=1, Nq=137, Nk=211, Hq=2, Hkv=2, d=64, causal=False, seed=16500)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    pad = 4096

    def guarded(like):
        buf = torch.full((like.numel() + 2 * pad,), 7.0, dtype=torch.bfloat16, device="cuda")
        return buf, buf[pad:pad + like.numel()].view(like.shape)

    bO, O = guarded(Q)
    bQ, dQ = guarded(Q)
    bK, dK = guarded(K)
    bV, dV = guarded(V)
    O, L = binding.fa_local_fwd(Q, K, V, prob.scale, 20, 3, O=O)
    binding.fa_local_bwd(Q, K, V, O, dO, L, prob.scale, 20, 3, dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    for buf in (bO, bQ, bK, bV):
        assert bool((buf[:pad] == 7.0).all()) and bool((buf[-pad:] == 7.0).all())
    for t in (O, L, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()


def test_bad_windows_and_shapes_are_rejected():
    q = torch.zeros(1, 32, 2, 64, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(1, 16, 2, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.FaError) as e:
        binding.fa_local_fwd(q, k, k, 0.125, 4, 0)   # more queries than keys
    assert e.value.status == binding.FA_ERR_SHAPE
    q96 = torch.zeros(1, 32, 2, 96, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.FaError) as e:
        binding.fa_local_fwd(q96, q96, q96, 0.1, 4, 0)
    assert e.value.status == binding.FA_ERR_UNSUPPORTED
    binding.fa_local_fwd(q96, q96, q96, 0.1, -1, 0)  # reduces to causal attention: any supported d
    torch.cuda.synchronize()


@pytest.mark.parametrize("name,left,right", [("d128_n8k_causal", 1023, 0), ("sweep_d64_n8192_full", 500, 500)])
def test_full_size_window_sampled_units(name, left, right):
    prob = inputs.make_config(name)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    O, L = binding.fa_local_fwd(Q, K, V, prob.scale, left, right)
    dQ, dK, dV = binding.fa_local_bwd(Q, K, V, O, dO, L, prob.scale, left, right)
    torch.cuda.synchronize()
    for t in (O, L, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()
    vis = orc.window_visible(prob.N, prob.N, left, right)
    M = window_mask_gpu(prob.N, prob.N, left, right)[0, 0]
    for (b, h) in ((0, 0), (prob.B - 1, prob.Hq - 1)):
        q, k, v, do = (orc.widen_bf16(x[b, :, h]) for x in (prob.Q, prob.K, prob.V, prob.dO))
        o, lse, _ = orc.head_forward_pattern(q, k, v, vis, prob.scale)
        dq, dk, dv = orc.head_backward_pattern(q, k, v, vis, do, prob.scale)
        ref = pu.reference_head(Q[b, :, h], K[b, :, h], V[b, :, h], dO[b, :, h], prob.scale, False, M=M)
        pu.judge(f"window ({left},{right}) {name} unit ({b},{h})",
                 {nm: pu.to_f64(t) for nm, t in (("O", O[b, :, h]), ("LSE", L[b, h]), ("dQ", dQ[b, :, h]), ("dK", dK[b, :, h]),
                                                 ("dV", dV[b, :, h]))},
                 dict(O=o, LSE=lse, dQ=dq, dK=dk, dV=dv), ref, d=prob.d)
