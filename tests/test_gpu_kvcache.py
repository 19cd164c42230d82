"""GPU parity for fa_kvcache_fwd (queries against a key/value cache with per-sequence lengths,
contiguous or paged) against the float64 oracle's kvcache_forward: lengths of 0, 1, a ragged tail
and the full capacity in one batch; one query and several; grouped heads; page sizes of one, two
and four key blocks with the pages shuffled in their pools; slack rows and unused pages filled
with NaN (never read); the reductions to the split-key entry point."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402


def draw(seed, B, Nq, cap, Hq, Hkv, d):
    prob = inputs.make_cross(B=B, Nq=Nq, Nk=cap, Hq=Hq, Hkv=Hkv, d=d, causal=False, seed=seed)
    return prob


def reference(Q, K_of, V_of, lens, scale, causal, Hq, Hkv):
    """The 16-bit materialising reference, sequence by sequence on the keys each one holds."""
    B, Nq = Q.shape[0], Q.shape[1]
    out = {"O": np.zeros(tuple(Q.shape)), "LSE": np.full((B, Hq, Nq), -np.inf)}
    G = Hq // Hkv
    for b in range(B):
        if lens[b] == 0:
            continue
        k, v = K_of(b), V_of(b)
        for h in range(Hq):
            r = pu.reference_head(Q[b, :, h], k[:, h // G], v[:, h // G], None, scale, causal, backward=False)
            out["O"][b, :, h], out["LSE"][b, h] = r["O"], r["LSE"]
    return out


def check_contiguous(prob, lens, causal, num_splits):
    Q, Kc, Vc = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V))
    cap = Kc.shape[1]
    for b, n in enumerate(lens):  # what lies past a sequence's length is not part of it
        Kc[b, n:] = float("nan")
        Vc[b, n:] = float("nan")
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    O, L = binding.fa_kvcache_fwd(Q, Kc, Vc, prob.scale, causal, seqlens_k=sl, num_splits=num_splits)
    torch.cuda.synchronize()
    Qf, Kf, Vf = (orc.widen_bf16(x) for x in (prob.Q, prob.K, prob.V))
    eO, eL = orc.kvcache_forward(Qf, Kf, Vf, prob.scale, causal, np.asarray(lens))
    ref = reference(Q, lambda b: Kc[b, :lens[b]], lambda b: Vc[b, :lens[b]], lens, prob.scale, causal, prob.Hq, prob.Hkv)
    pu.judge(f"cache {lens} of {cap} Nq{prob.N} H{prob.Hq}/{prob.Hkv} d{prob.d} {'c' if causal else 'f'} x{num_splits}",
             {"O": pu.to_f64(O), "LSE": pu.to_f64(L)}, {"O": eO, "LSE": eL}, ref, d=prob.d)
    return O, L


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("num_splits", [1, 3, 0])
@pytest.mark.parametrize("Nq,Hq,Hkv,d", [(1, 8, 2, 128), (1, 4, 4, 64), (3, 8, 1, 128), (70, 4, 2, 64)])
def test_contiguous_cache_with_lengths(Nq, Hq, Hkv, d, num_splits, causal):
    cap = 1000
    check_contiguous(draw(18000 + Nq + d, 5, Nq, cap, Hq, Hkv, d), [cap, 1, 0, 517, 64], causal, num_splits)


def page_out(Kc, Vc, lens, page, seed, spare=3):
    """Cut contiguous caches [B, cap, Hkv, d] into pages that lie shuffled in pools with `spare` pages
    nobody owns; pages that a sequence does not reach, the spare ones and the slack of every last
    page hold NaN. Returns the pools and the table (unreached entries name a spare page)."""
    B, cap = Kc.shape[0], Kc.shape[1]
    pps = -(-cap // page)
    g = np.random.default_rng(seed)
    perm = g.permutation(B * pps + spare)
    table = perm[:B * pps].reshape(B, pps).copy()
    Kp = torch.full((B * pps + spare, page) + tuple(Kc.shape[2:]), float("nan"), dtype=Kc.dtype, device=Kc.device)
    Vp = torch.full_like(Kp, float("nan"))
    for b in range(B):
        for i in range(pps):
            lo, hi = i * page, min((i + 1) * page, lens[b])
            if hi > lo:
                Kp[table[b, i], :hi - lo] = Kc[b, lo:hi]
                Vp[table[b, i], :hi - lo] = Vc[b, lo:hi]
            else:
                table[b, i] = perm[B * pps + (b + i) % spare]
    return Kp, Vp, torch.from_numpy(table.astype(np.int32)).cuda()


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("page", [64, 128, 256])
@pytest.mark.parametrize("Nq,Hq,Hkv,d,num_splits", [(1, 8, 2, 128, 0), (1, 4, 4, 64, 2), (5, 8, 1, 128, 3), (70, 4, 2, 64, 1)])
def test_paged_cache(Nq, Hq, Hkv, d, num_splits, page, causal):
    cap, lens = 1024, [1024, 1, 0, 517, 64, 700]
    prob = draw(18100 + Nq + d + page, len(lens), Nq, cap, Hq, Hkv, d)
    Q, Kc, Vc = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V))
    Kp, Vp, table = page_out(Kc, Vc, lens, page, 18200 + page)
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    O, L = binding.fa_kvcache_fwd(Q, Kp, Vp, prob.scale, causal, seqlens_k=sl, block_table=table, num_splits=num_splits)
    torch.cuda.synchronize()
    Qf, Kf, Vf = (orc.widen_bf16(x) for x in (prob.Q, prob.K, prob.V))
    tab = table.cpu().numpy()
    Kpool = np.zeros((Kp.shape[0], page, Hkv, d))
    Vpool = np.zeros_like(Kpool)
    for b in range(len(lens)):  # the oracle's pools: the same pages, from the float64 tensors
        for i in range(tab.shape[1]):
            lo, hi = i * page, min((i + 1) * page, lens[b])
            if hi > lo:
                Kpool[tab[b, i], :hi - lo] = Kf[b, lo:hi]
                Vpool[tab[b, i], :hi - lo] = Vf[b, lo:hi]
    eO, eL = orc.kvcache_forward(Qf, Kpool, Vpool, prob.scale, causal, np.asarray(lens), tab)
    ref = reference(Q, lambda b: Kc[b, :lens[b]], lambda b: Vc[b, :lens[b]], lens, prob.scale, causal, Hq, Hkv)
    pu.judge(f"paged cache page {page} Nq{Nq} H{Hq}/{Hkv} d{d} {'c' if causal else 'f'} x{num_splits}",
             {"O": pu.to_f64(O), "LSE": pu.to_f64(L)}, {"O": eO, "LSE": eL}, ref, d=d)
    # the same keys in one slab per sequence: the same arithmetic in the same order
    O2, L2 = binding.fa_kvcache_fwd(Q, Kc, Vc, prob.scale, causal, seqlens_k=sl,
                                    num_splits=num_splits or binding.splitkv_default_splits(len(lens), Hq, Hkv, Nq, cap, ragged=True))
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and torch.equal(L, L2)


def test_full_lengths_reproduce_the_split_key_entry_point_bitwise():
    prob = draw(18300, 3, 2, 700, 8, 2, 128)
    Q, Kc, Vc = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V))
    for causal in (False, True):
        O1, L1 = binding.fa_kvcache_fwd(Q, Kc, Vc, prob.scale, causal, num_splits=4)
        sl = torch.full((3,), 700, dtype=torch.int32, device="cuda")
        O2, L2 = binding.fa_kvcache_fwd(Q, Kc, Vc, prob.scale, causal, seqlens_k=sl, num_splits=4)
        O3, L3 = binding.fa_splitkv_fwd(Q, Kc, Vc, prob.scale, causal, num_splits=4)
        torch.cuda.synchronize()
        assert torch.equal(O1, O3) and torch.equal(L1, L3) and torch.equal(O2, O3) and torch.equal(L2, L3)


def test_more_queries_than_cached_keys_under_the_causal_rule():
    """Rows that stand before the first key see nothing: O = 0, LSE = -inf; the others are exact."""
    check_contiguous(draw(18400, 3, 40, 300, 4, 2, 128), [10, 40, 300], True, 2)


def test_a_decode_batch_at_full_size_sampled_sequences():
    """64 sequences, one query each, 32 query heads on 8 key/value heads, lengths up to 8192 in pages of 256."""
    B, cap, Hq, Hkv, d, page = 64, 8192, 32, 8, 128, 256
    g = np.random.default_rng(18500)
    lens = [int(x) for x in g.integers(1, cap + 1, B)]
    lens[0], lens[1] = cap, 1
    prob = draw(18501, B, 1, cap, Hq, Hkv, d)
    Q, Kc, Vc = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V))
    Kp, Vp, table = page_out(Kc, Vc, lens, page, 18502)
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    O, L = binding.fa_kvcache_fwd(Q, Kp, Vp, prob.scale, False, seqlens_k=sl, block_table=table)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all() and torch.isfinite(L).all()
    for b in (0, 1, 17, B - 1):
        q, k, v = orc.widen_bf16(prob.Q[b:b + 1]), orc.widen_bf16(prob.K[b:b + 1, :lens[b]]), orc.widen_bf16(prob.V[b:b + 1, :lens[b]])
        eO, eL = orc.attention_forward(q, k, v, prob.scale, False)
        ref = reference(Q[b:b + 1], lambda _: Kc[b, :lens[b]], lambda _: Vc[b, :lens[b]], [lens[b]], prob.scale, False, Hq, Hkv)
        pu.judge(f"decode batch, sequence {b} ({lens[b]} keys)", {"O": pu.to_f64(O[b:b + 1]), "LSE": pu.to_f64(L[b:b + 1])},
                 {"O": eO, "LSE": eL}, ref, d=d)


def test_bad_cache_descriptions_are_rejected():
    q = torch.zeros(2, 1, 4, 64, dtype=torch.bfloat16, device="cuda")
    pool = torch.zeros(8, 32, 4, 64, dtype=torch.bfloat16, device="cuda")  # pages of 32 rows: not whole key blocks
    table = torch.zeros(2, 4, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.FaError) as e:
        binding.fa_kvcache_fwd(q, pool, pool, 0.125, False, block_table=table)
    assert e.value.status == binding.FA_ERR_UNSUPPORTED
    pool = torch.zeros(8, 64, 4, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.FaError) as e:
        binding.fa_kvcache_fwd(q, pool, pool, 0.125, False, block_table=table, max_seqlen_k=300)  # 4 pages hold 256
    assert e.value.status == binding.FA_ERR_SHAPE
    with pytest.raises(ValueError):
        binding.fa_kvcache_fwd(q, pool, pool, 0.125, False, block_table=table.long())
    with pytest.raises(ValueError):
        binding.fa_kvcache_fwd(q, pool, pool, 0.125, False, seqlens_k=torch.zeros(3, dtype=torch.int32, device="cuda"),
                               block_table=table)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Nq,Hq,Hkv", [(4, 8, 1), (32, 2, 2), (16, 4, 2), (33, 1, 1), (5, 8, 1), (1, 32, 1)])
def test_row_counts_around_the_decode_kernel_limit(Nq, Hq, Hkv, d, causal):
    """Nq * (Hq / Hkv) = 32 rows per key/value head is the most the decode kernel takes (one MFMA row
    tile); 33 and 40 go to the row-block kernel. Lengths from one key to the capacity, more shares
    than some sequences have key blocks (empty shares), a length that ends inside a 32-key tile."""
    cap, lens = 2000, [2000, 1, 33, 95, 1024, 0, 1999]
    check_contiguous(draw(18600 + Nq + Hq + d, len(lens), Nq, cap, Hq, Hkv, d), lens, causal, 7)


@pytest.mark.parametrize("B", [2, 64, 128, 129])
def test_many_sequences_with_equal_and_uneven_lengths(B):
    """The decode kernel hands up to 128 sequences out longest first (a rank per workgroup, ties by
    index); 129 keep the launch order. Lengths with many ties, zeros among them."""
    cap, Hq, Hkv, d = 256, 4, 2, 64
    g = np.random.default_rng(18700 + B)
    lens = [int(x) for x in g.choice([0, 1, 64, 64, 100, 256, 256, 255], B)]
    check_contiguous(draw(18701 + B, B, 1, cap, Hq, Hkv, d), lens, True, 2)


def test_decoding_steps_replay_from_a_captured_graph():
    """A serving loop captures one decoding step into a HIP graph and replays it while the cache grows:
    the lengths, the page table and the cache contents live in device buffers that change between
    replays, the launch itself does not. Every replay must give the eager result bit for bit."""
    B, cap, Hq, Hkv, d, page = 6, 1024, 8, 2, 128, 128
    prob = draw(18800, B, 1, cap, Hq, Hkv, d)
    Q, Kc, Vc = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V))
    lens = [1000, 1, 300, 64, 0, 777]
    Kp, Vp, table = page_out(Kc, Vc, [cap] * B, page, 18801)
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    splits = 2
    O = torch.empty_like(Q)
    L = torch.empty(B, Hq, 1, device="cuda")
    ws = torch.empty(binding.fa_splitkv_fwd_workspace_bytes(B, Hq, 1, d, splits), dtype=torch.uint8, device="cuda")

    def step():
        binding.fa_kvcache_fwd(Q, Kp, Vp, prob.scale, True, seqlens_k=sl, block_table=table, num_splits=splits, O=O, LSE=L,
                               workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for trial in range(4):
        if trial:  # the batch moves on: longer caches, new queries, pages that changed hands
            sl.copy_(torch.clamp(sl + 17 * trial, max=cap))
            Q.copy_(torch.randn_like(Q))
            table.copy_(table.flip(0) if trial == 2 else table)
        step()
        torch.cuda.synchronize()
        eager = [O.clone(), L.clone()]
        O.fill_(float("nan"))
        L.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(eager[0], O) and torch.equal(eager[1], L)
