"""GPU parity for the elementwise mask added to the scores (fa_mask_fwd / fa_mask_bwd) against
the float64 oracle: biases, boolean masks, rows left without any key, masks shared over batch
and heads, ragged lengths on both sides, with and without the causal rule."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402


def make_mask(seed, Bm, Hm, Nq, Nk, kind, dtype="bf16"):
    """Mask values as bit patterns of the element type [Bm, Hm, Nq, Nk]: 'bias' N(0, 2^2); 'bool' 0 / -inf with
    30 % removed; 'mixed' bias with 30 % removed; key 0 always stays (every row keeps one entry,
    also under the causal rule). 'dead' additionally removes whole rows."""
    g = np.random.default_rng(seed)
    m = np.zeros((Bm, Hm, Nq, Nk), dtype=np.float32) if kind == "bool" else \
        (2.0 * g.standard_normal((Bm, Hm, Nq, Nk))).astype(np.float32)
    if kind != "bias":
        gone = g.random((Bm, Hm, Nq, Nk)) < 0.3
        gone[..., 0] = False
        m[gone] = -np.inf
    if kind == "dead":
        rows = g.random((Bm, Hm, Nq)) < 0.2
        m[rows] = -np.inf
    return inputs.f32_to_f16_bits(m) if dtype == "f16" else inputs.f32_to_bf16_bits(m)


def mask_to_gpu(bits, dtype="bf16"):
    Bm, Hm, Nq, Nk = bits.shape
    M = binding.mask_buffer(Bm, Hm, Nq, Nk, dtype=torch.float16 if dtype == "f16" else torch.bfloat16)
    M.copy_(pu.to_gpu(bits, dtype))
    return M


def check_mask(prob, mbits, fwd_only=False):
    Q, K, V, dO = (pu.to_gpu(x, prob.dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    M = mask_to_gpu(mbits, prob.dtype)
    O, L = binding.fa_mask_fwd(Q, K, V, M, prob.scale, prob.causal)
    widen = orc.widen_f16 if prob.dtype == "f16" else orc.widen_bf16
    Qf, Kf, Vf, dOf, Mf = (widen(x) for x in (prob.Q, prob.K, prob.V, prob.dO, mbits))
    eO, eL = orc.attention_forward_masked(Qf, Kf, Vf, Mf, prob.scale, prob.causal)
    got = {"O": O, "LSE": L}
    exp = {"O": eO, "LSE": eL}
    if not fwd_only:
        dQ, dK, dV = binding.fa_mask_bwd(Q, K, V, M, O, dO, L, prob.scale, prob.causal)
        got.update(dQ=dQ, dK=dK, dV=dV)
        exp.update(zip(("dQ", "dK", "dV"), orc.attention_backward_masked(Qf, Kf, Vf, Mf, dOf, prob.scale, prob.causal)))
    torch.cuda.synchronize()
    Bm, Hm, Nq, Nk = mbits.shape
    ref = pu.reference_batch(Q, K, V, dO, prob.scale, prob.causal, backward=not fwd_only, M=M[:, :, :, :Nk])
    res = pu.judge(f"mask {pu.describe(prob)} shared {Bm}x{Hm}", {k: pu.to_f64(v) for k, v in got.items()}, exp, ref,
                   dtype=prob.dtype, d=prob.d)
    return {k: v[0] for k, v in res.items()}


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("kind", ["bias", "bool", "mixed"])
@pytest.mark.parametrize("N", [1, 65, 300, 515])
def test_masked_self_attention(N, kind, d, causal):
    prob = inputs.make_dense(B=2, N=N, Hq=2, Hkv=2, d=d, causal=causal, seed=9000 + N)
    check_mask(prob, make_mask(9100 + N, 2, 2, N, N, kind))


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("kind", ["bias", "mixed", "dead"])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d", [(65, 65, 2, 2, 64), (70, 333, 4, 2, 128), (300, 515, 2, 1, 64), (515, 515, 2, 2, 128)])
def test_masks_in_half_precision(Nq, Nk, Hq, Hkv, d, kind, causal):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=9050 + Nq + Nk, dtype="f16")
    check_mask(prob, make_mask(9060 + Nq, 2, Hq, Nq, Nk, kind, dtype="f16"))


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d", [(70, 333, 4, 2, 128), (1, 300, 8, 2, 64), (300, 301, 4, 1, 128),
                                            (257, 1000, 2, 2, 64), (300, 129, 2, 2, 128)])
def test_two_lengths_and_grouped_heads(Nq, Nk, Hq, Hkv, d, causal):
    if causal and Nq > Nk:
        pytest.skip("causal needs at least as many keys as queries")
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=9200 + Nq)
    check_mask(prob, make_mask(9300 + Nq, 2, Hq, Nq, Nk, "mixed"))


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
def test_rows_left_without_any_key(d, causal):
    prob = inputs.make_cross(B=2, Nq=200, Nk=330, Hq=4, Hkv=2, d=d, causal=causal, seed=9400 + d)
    mbits = make_mask(9401, 2, 4, 200, 330, "dead")
    check_mask(prob, mbits)
    # the outputs of such rows are exactly zero
    dead = np.all(np.isneginf(orc.widen_bf16(mbits)), axis=3)  # [B, Hq, Nq]
    assert dead.any()
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    M = mask_to_gpu(mbits)
    O, L = binding.fa_mask_fwd(Q, K, V, M, prob.scale, causal)
    dQ, _, _ = binding.fa_mask_bwd(Q, K, V, M, O, dO, L, prob.scale, causal)
    torch.cuda.synchronize()
    sel = torch.from_numpy(dead.transpose(0, 2, 1).copy()).cuda()  # [B, Nq, Hq]
    assert not bool(O[sel].any()) and not bool(dQ[sel].any())


@pytest.mark.parametrize("Bm,Hm", [(1, 1), (2, 1), (1, 4)])
def test_masks_shared_over_sequences_and_heads(Bm, Hm):
    prob = inputs.make_cross(B=2, Nq=130, Nk=200, Hq=4, Hkv=2, d=128, causal=False, seed=9500)
    check_mask(prob, make_mask(9501 + Bm + Hm, Bm, Hm, 130, 200, "mixed"))


def test_a_zero_mask_reproduces_the_plain_entry_points():
    prob = inputs.make_cross(B=2, Nq=300, Nk=301, Hq=4, Hkv=2, d=128, causal=True, seed=9600)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    M = binding.mask_buffer(1, 1, 300, 301)
    O1, L1 = binding.fa_cross_fwd(Q, K, V, prob.scale, True)
    O2, L2 = binding.fa_mask_fwd(Q, K, V, M, prob.scale, True)
    g1 = binding.fa_cross_bwd(Q, K, V, O1, dO, L1, prob.scale, True)
    g2 = binding.fa_mask_bwd(Q, K, V, M, O1, dO, L1, prob.scale, True)
    torch.cuda.synchronize()
    # same arithmetic up to the order of two roundings in the exponent
    assert float((O1.float() - O2.float()).abs().max()) <= 2e-3
    assert float((L1 - L2).abs().max()) <= 1e-5
    for a, b in zip(g1, g2):
        assert float((a.float() - b.float()).abs().max()) <= 4e-3 * max(1.0, float(a.float().abs().max()))


def test_the_causal_rule_written_as_a_mask():
    prob = inputs.make_dense(B=1, N=400, Hq=2, Hkv=2, d=64, causal=False, seed=9700)
    Q, K, V = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V))
    M = binding.mask_buffer(1, 1, 400, 400)
    M.masked_fill_(torch.ones(400, 400, dtype=torch.bool, device="cuda").triu(1), float("-inf"))
    O1, L1 = binding.fa_fwd(Q, K, V, prob.scale, True)
    O2, L2 = binding.fa_mask_fwd(Q, K, V, M, prob.scale, False)
    torch.cuda.synchronize()
    assert float((O1.float() - O2.float()).abs().max()) <= 2e-3
    assert float((L1 - L2).abs().max()) <= 1e-5


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d,kind,Bm,Hm", [(65, 65, 2, 2, 64, "bias", 2, 2), (70, 333, 4, 2, 128, "mixed", 2, 4),
                                                       (300, 515, 2, 1, 64, "dead", 2, 2), (515, 515, 4, 2, 128, "mixed", 1, 1),
                                                       (257, 300, 2, 2, 128, "bias", 2, 1)])
def test_gradient_of_the_mask(Nq, Nk, Hq, Hkv, d, kind, Bm, Hm, dtype, causal):
    """fa_mask_bwd_dmask: dM = dS for every (sequence, head), also under shared masks, against the
    oracle's mask gradient and the 16-bit reference's dS; dQ, dK, dV are those of fa_mask_bwd bit for bit;
    the padding of dM's rows holds nothing but zeros; entries the mask or the causal rule removes are 0."""
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=9300 + Nq + Nk, dtype=dtype)
    mbits = make_mask(9310 + Nq, Bm, Hm, Nq, Nk, kind, dtype=dtype)
    Q, K, V, dO = (pu.to_gpu(x, dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    M = mask_to_gpu(mbits, dtype)
    O, L = binding.fa_mask_fwd(Q, K, V, M, prob.scale, causal)
    dQ, dK, dV, dM = binding.fa_mask_bwd_dmask(Q, K, V, M, O, dO, L, prob.scale, causal)
    g2 = binding.fa_mask_bwd(Q, K, V, M, O, dO, L, prob.scale, causal)
    torch.cuda.synchronize()
    for a, b in zip((dQ, dK, dV), g2):
        assert torch.equal(a, b)
    widen = orc.widen_f16 if dtype == "f16" else orc.widen_bf16
    Qf, Kf, Vf, dOf, Mf = (widen(x) for x in (prob.Q, prob.K, prob.V, prob.dO, mbits))
    Mfull = np.broadcast_to(Mf, (2, Hq, Nq, Nk))
    exp = orc.attention_backward_mask_gradient(Qf, Kf, Vf, Mfull, dOf, prob.scale, causal)
    ref = pu.reference_batch(Q, K, V, dO, prob.scale, causal, M=M[:, :, :, :Nk], want_dm=True)
    # (no fixed bound is stated for dM anywhere: the yardstick clause alone, error <= the 16-bit reference's + 1 ulp)
    pu.judge(f"mask gradient {pu.describe(prob)} {kind} shared {Bm}x{Hm}", {"dM": pu.to_f64(dM)}, {"dM": exp}, ref,
             standard=False, dtype=dtype, d=d)
    gone = np.isneginf(Mfull) | (causal & (np.arange(Nk)[None, :] > np.arange(Nq)[:, None] + Nk - Nq))[None, None]
    assert not pu.to_f64(dM)[gone].any()
    whole = dM.as_strided((2, Hq, Nq, dM.stride(2)), (dM.stride(0), dM.stride(1), dM.stride(2), 1))
    assert not whole[..., Nk:].float().abs().any()


def test_bad_mask_descriptions_are_rejected():
    q = torch.zeros(1, 16, 2, 64, dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q)
    lse = torch.empty(1, 2, 16, dtype=torch.float32, device="cuda")
    m = torch.zeros(1, 1, 16, 16, dtype=torch.bfloat16, device="cuda")
    args = (q.data_ptr(), q.data_ptr(), q.data_ptr())

    def run(M=m.data_ptr(), bs=0, hs=0, rs=16, d=64):
        return binding.fa_mask_fwd_raw(*args, M, o.data_ptr(), lse.data_ptr(), 1, 2, 2, 16, 16, d, 0.125, 0, bs, hs, rs, 0)
    assert run() == binding.FA_OK
    assert run(M=0) == binding.FA_ERR_NULL
    assert run(M=m.data_ptr() + 2) == binding.FA_ERR_ALIGN
    assert run(rs=8) == binding.FA_ERR_SHAPE     # shorter than a row
    assert run(rs=20) == binding.FA_ERR_SHAPE    # not a multiple of 8
    assert run(hs=-8) == binding.FA_ERR_SHAPE
    assert run(bs=4) == binding.FA_ERR_SHAPE
    torch.cuda.synchronize()


@pytest.mark.timeout(600)
def test_full_size_masked_workload_sampled_units():
    """The shape of the benchmark workload (B=2, N=8192, 16 heads of 128, causal) with one mask per
    head shared by the two sequences: 30 % of the entries removed, a bias on the rest. The mask is
    drawn on the GPU; whole (sequence, head) units are compared with the oracle."""
    prob = inputs.make_config("d128_n8k_causal")
    B, N, H = prob.B, prob.N, prob.Hq
    gen = torch.Generator(device="cuda").manual_seed(9800)
    M = binding.mask_buffer(1, H, N, N)
    M.copy_(2.0 * torch.randn(1, H, N, N, device="cuda", generator=gen))
    gone = torch.rand(1, H, N, N, device="cuda", generator=gen) < 0.3
    gone[..., 0] = False
    M.masked_fill_(gone, float("-inf"))
    del gone
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    O, L = binding.fa_mask_fwd(Q, K, V, M, prob.scale, True)
    dQ, dK, dV = binding.fa_mask_bwd(Q, K, V, M, O, dO, L, prob.scale, True)
    torch.cuda.synchronize()
    for t in (O, L, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()
    for (b, h) in ((0, 0), (B - 1, H - 1)):
        q, k, v, do = (orc.widen_bf16(x[b, :, h]) for x in (prob.Q, prob.K, prob.V, prob.dO))
        m = M[0, h].double().cpu().numpy()
        o, lse, _ = orc.head_forward_masked(q, k, v, m, prob.scale, True)
        dq, dk, dv = orc.head_backward_masked(q, k, v, m, do, prob.scale, True)
        ref = pu.reference_head(Q[b, :, h], K[b, :, h], V[b, :, h], dO[b, :, h], prob.scale, True, M=M[0, h, :, :N])
        pu.judge(f"masked {prob.name} unit ({b},{h})",
                 {nm: pu.to_f64(t) for nm, t in (("O", O[b, :, h]), ("LSE", L[b, h]), ("dQ", dQ[b, :, h]), ("dK", dK[b, :, h]),
                                                 ("dV", dV[b, :, h]))},
                 dict(O=o, LSE=lse, dQ=dq, dK=dk, dV=dv), ref, d=prob.d)
