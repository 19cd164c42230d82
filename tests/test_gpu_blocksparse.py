"""GPU parity for block-sparse attention, fa_blocksparse_fwd / fa_blocksparse_bwd, against the
float64 oracle's block pattern: random patterns at several densities and block sizes, with and
without the causal rule, row blocks left without any key (exact zeros, L = -inf), patterns shared
over sequences and heads, grouped heads, two lengths, ragged tails; the full pattern against the
plain entry points; a full-size workload on sampled units."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402


def draw_pattern(seed, Bm, Hm, nq, nk, block, density, keep_first=True):
    g = np.random.default_rng(seed)
    bm = g.random((Bm, Hm, -(-nq // block), -(-nk // block))) < density
    if keep_first:
        bm[..., 0] = True  # every row block keeps key block 0 (visible under the causal rule as well)
    return bm


def additive_mask_gpu(bm, nq, nk, block):
    """The block pattern as an additive mask [Bm, Hm, nq, nk] (0 / -inf) for the 16-bit reference."""
    t = torch.from_numpy(bm).cuda()
    vis = t.repeat_interleave(block, dim=2).repeat_interleave(block, dim=3)[:, :, :nq, :nk]
    return torch.where(vis, 0.0, float("-inf"))


def check_blocksparse(prob, bm, block):
    Q, K, V, dO = (pu.to_gpu(x, prob.dtype) for x in (prob.Q, prob.K, prob.V, prob.dO))
    BM = torch.from_numpy(bm.astype(np.uint8)).cuda()
    O, L = binding.fa_blocksparse_fwd(Q, K, V, BM, block, prob.scale, prob.causal)
    dQ, dK, dV = binding.fa_blocksparse_bwd(Q, K, V, BM, block, O, dO, L, prob.scale, prob.causal)
    torch.cuda.synchronize()
    widen = orc.widen_f16 if prob.dtype == "f16" else orc.widen_bf16
    Qf, Kf, Vf, dOf = (widen(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    exp = {}
    exp["O"], exp["LSE"] = orc.attention_forward_blocksparse(Qf, Kf, Vf, prob.scale, prob.causal, bm, block)
    exp["dQ"], exp["dK"], exp["dV"] = orc.attention_backward_blocksparse(Qf, Kf, Vf, dOf, prob.scale, prob.causal, bm, block)
    ref = pu.reference_batch(Q, K, V, dO, prob.scale, prob.causal, M=additive_mask_gpu(bm, prob.N, prob.keys, block))
    pu.judge(f"block pattern {block} {bm.shape[0]}x{bm.shape[1]} {pu.describe(prob)}",
             {nm: pu.to_f64(t) for nm, t in (("O", O), ("LSE", L), ("dQ", dQ), ("dK", dK), ("dV", dV))}, exp, ref,
             dtype=prob.dtype, d=prob.d)
    return O, L, dQ, dK, dV


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Nq,Nk,block,density", [(300, 300, 64, 0.5), (700, 700, 128, 0.5), (300, 1000, 64, 0.3), (1100, 1100, 256, 0.5)])
def test_patterns_in_half_precision(Nq, Nk, block, density, d, causal):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=4, Hkv=2, d=d, causal=causal, seed=17050 + Nq + Nk, dtype="f16")
    check_blocksparse(prob, draw_pattern(17060 + Nq, 2, 4, Nq, Nk, block, density), block)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("N,block,density", [(64, 64, 1.0), (300, 64, 0.5), (700, 64, 0.3), (700, 128, 0.5), (1100, 256, 0.5),
                                             (1100, 64, 0.15), (515, 512, 0.7)])
def test_random_patterns(N, block, density, d, causal):
    prob = inputs.make_dense(B=2, N=N, Hq=2, Hkv=2, d=d, causal=causal, seed=17000 + N + block)
    check_blocksparse(prob, draw_pattern(17100 + N, 2, 2, N, N, block, density), block)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
def test_row_blocks_without_any_key(d, causal):
    prob = inputs.make_dense(B=2, N=600, Hq=2, Hkv=2, d=d, causal=causal, seed=17200 + d)
    bm = draw_pattern(17201, 2, 2, 600, 600, 64, 0.4)
    bm[0, 0, 3] = False   # rows 192 .. 255 of the first unit see nothing
    bm[1, 1, 0] = False   # and the first rows of the last one
    bm[:, :, 9] = False   # the ragged last row block everywhere
    O, L, dQ, dK, dV = check_blocksparse(prob, bm, 64)
    assert not bool(O[0, 192:256, 0].any()) and not bool(dQ[0, 192:256, 0].any()) and bool(torch.isneginf(L[0, 0, 192:256]).all())
    assert not bool(O[:, 576:].any()) and not bool(dQ[:, 576:].any())


@pytest.mark.parametrize("Bm,Hm", [(1, 1), (2, 1), (1, 4)])
def test_patterns_shared_over_sequences_and_heads_grouped_heads(Bm, Hm):
    prob = inputs.make_cross(B=2, Nq=400, Nk=400, Hq=4, Hkv=2, d=128, causal=True, seed=17300)
    check_blocksparse(prob, draw_pattern(17301 + Bm + Hm, Bm, Hm, 400, 400, 128, 0.5), 128)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Nq,Nk,Hq,Hkv,d,block", [(70, 333, 4, 2, 128, 64), (300, 1000, 8, 2, 64, 128), (257, 300, 2, 1, 128, 64),
                                                  (1, 300, 2, 2, 64, 64)])
def test_two_lengths(Nq, Nk, Hq, Hkv, d, block, causal):
    prob = inputs.make_cross(B=2, Nq=Nq, Nk=Nk, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=17400 + Nq)
    # (two lengths under the causal rule: the first key block need not be visible to every row; keep the diagonal too)
    bm = draw_pattern(17401 + Nq, 2, Hq, Nq, Nk, block, 0.5)
    if causal:
        for rb in range(bm.shape[2]):
            bm[:, :, rb, min((rb * block + Nk - Nq) // block, bm.shape[3] - 1)] = True
    check_blocksparse(prob, bm, block)


def test_the_full_pattern_is_plain_attention():
    prob = inputs.make_cross(B=2, Nq=300, Nk=420, Hq=4, Hkv=2, d=128, causal=True, seed=17500)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    BM = torch.ones(1, 1, 5, 7, dtype=torch.uint8, device="cuda")
    O1, L1 = binding.fa_blocksparse_fwd(Q, K, V, BM, 64, prob.scale, True)
    O2, L2 = binding.fa_cross_fwd(Q, K, V, prob.scale, True)
    g1 = binding.fa_blocksparse_bwd(Q, K, V, BM, 64, O1, dO, L1, prob.scale, True)
    g2 = binding.fa_cross_bwd(Q, K, V, O2, dO, L2, prob.scale, True)
    torch.cuda.synchronize()
    assert float((O1.float() - O2.float()).abs().max()) <= 2 * pu.bf16_ulp(float(O2.float().abs().max()))
    assert float((L1 - L2).abs().max()) <= 1e-5
    for a, b in zip(g1, g2):
        assert float((a.float() - b.float()).abs().max()) <= 2 * pu.bf16_ulp(float(b.float().abs().max()))


def test_bad_patterns_are_rejected():
    q = torch.zeros(1, 128, 2, 64, dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q)
    lse = torch.empty(1, 2, 128, dtype=torch.float32, device="cuda")
    bm = torch.ones(1, 1, 2, 2, dtype=torch.uint8, device="cuda")
    p = q.data_ptr()

    def run(BM=bm.data_ptr(), block=64, bs=0, hs=0, d=64):
        return binding.fa_blocksparse_fwd_raw(p, p, p, BM, o.data_ptr(), lse.data_ptr(), 1, 2, 2, 128, 128, d, 0.125, 0, block, bs, hs, 0)
    assert run() == binding.FA_OK
    assert run(BM=0) == binding.FA_ERR_NULL
    assert run(block=32) == binding.FA_ERR_SHAPE
    assert run(block=96) == binding.FA_ERR_SHAPE
    assert run(block=0) == binding.FA_ERR_SHAPE
    assert run(hs=-4) == binding.FA_ERR_SHAPE
    assert run(d=96) == binding.FA_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    with pytest.raises(ValueError):
        binding.fa_blocksparse_fwd(q, q, q, torch.ones(1, 1, 3, 2, dtype=torch.uint8, device="cuda"), 64, 0.125, False)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d,block,density", [(128, 64, 0.1), (64, 64, 0.1), (128, 256, 0.2)])
def test_thin_patterns_with_long_visit_lists(d, block, density, causal):
    """Patterns thin enough that the workgroups walk their compacted lists of blocks, long enough that
    a list has a few hundred entries (4096 tokens, four query heads per key/value head: 512 row tiles
    per key block at d = 128), with a pattern of its own per query head."""
    prob = inputs.make_cross(B=1, Nq=4096, Nk=4096, Hq=4, Hkv=1, d=d, causal=causal, seed=17700 + d + block)
    check_blocksparse(prob, draw_pattern(17710 + d + block, 1, 4, 4096, 4096, block, density), block)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["blocksparse_d128_n8k_causal_half", "blocksparse_d128_n8k_causal_eighth"])
def test_full_size_pattern_sampled_units(name):
    """The benchmark shape (B=2, N=8192, 16 heads of 128, causal) under a pattern of 128 x 128 blocks,
    one per head, half (seven eighths) of the blocks below the diagonal removed; the diagonal and the
    first key block stay."""
    prob = inputs.make_config(name)
    N, block = prob.N, prob.meta["block_pattern"]["block"]
    bm = inputs.block_pattern(prob.meta["block_pattern"]["seed"], 1, prob.Hq, N, N, block, prob.meta["block_pattern"]["density"], True)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    BM = torch.from_numpy(bm.astype(np.uint8)).cuda()
    O, L = binding.fa_blocksparse_fwd(Q, K, V, BM, block, prob.scale, True)
    dQ, dK, dV = binding.fa_blocksparse_bwd(Q, K, V, BM, block, O, dO, L, prob.scale, True)
    torch.cuda.synchronize()
    for t in (O, L, dQ, dK, dV):
        assert torch.isfinite(t.float()).all()
    for (b, h) in ((0, 0), (prob.B - 1, prob.Hq - 1)):
        vis = orc.block_visible(N, N, bm[0, h], block)
        M = additive_mask_gpu(bm[:, h:h + 1], N, N, block)[0, 0]
        q, k, v, do = (orc.widen_bf16(x[b, :, h]) for x in (prob.Q, prob.K, prob.V, prob.dO))
        o, lse, _ = orc.head_forward_pattern(q, k, v, vis, prob.scale, True)
        dq, dk, dv = orc.head_backward_pattern(q, k, v, vis, do, prob.scale, True)
        ref = pu.reference_head(Q[b, :, h], K[b, :, h], V[b, :, h], dO[b, :, h], prob.scale, True, M=M)
        pu.judge(f"block pattern, {prob.name} unit ({b},{h})",
                 {nm: pu.to_f64(t) for nm, t in (("O", O[b, :, h]), ("LSE", L[b, h]), ("dQ", dQ[b, :, h]), ("dK", dK[b, :, h]),
                                                 ("dV", dV[b, :, h]))},
                 dict(O=o, LSE=lse, dQ=dq, dK=dk, dV=dv), ref, d=prob.d)
