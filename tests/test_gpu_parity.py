"""GPU parity: the HIP path, called through the C ABI binding, against the
float64 oracle on the same seeded bf16 inputs, element by element.

Bars (bf16 inputs ~ N(0,1)): max|dO| <= 2e-2, max|d(dQ,dK,dV)| <= 5e-2,
max|dLSE| <= 1e-3 against the oracle, and in every case the error must not
exceed that of a bf16 implementation that materialises S and P (section 2.2's
standard implementation) by more than one bf16 ulp at the tensor's largest
magnitude (parity_util.judge).
"""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs
from oracle import attention_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402


check = pu.check


def test_tiny_config_exact_shape():
    prob = inputs.make_config("tiny")
    errs = check(prob)
    print("tiny", errs)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("N", [1, 2, 31, 63, 64, 65, 127, 128, 129, 257, 300, 515])
def test_ragged_tail_lengths(N, d, causal):
    prob = inputs.make_dense(B=2, N=N, Hq=2, Hkv=2, d=d, causal=causal, seed=2000 + N)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d,Hq,Hkv", [(64, 4, 2), (128, 8, 2), (128, 4, 1), (64, 6, 6)])
def test_grouped_query_heads(d, Hq, Hkv, causal):
    prob = inputs.make_dense(B=2, N=200, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=2100 + Hq)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
def test_several_row_and_column_blocks(causal):
    prob = inputs.make_dense(B=1, N=1100, Hq=3, Hkv=3, d=128, causal=causal, seed=2200)
    check(prob)
    prob = inputs.make_dense(B=1, N=900, Hq=2, Hkv=1, d=64, causal=causal, seed=2201)
    check(prob)


def test_wide_score_range():
    # Q, K scaled by 3 before rounding: scores ~ N(0, 9^2 / sqrt(d) scale), LSE in the tens
    prob = inputs.make_dense(B=1, N=700, Hq=2, Hkv=2, d=128, causal=True, seed=2300, qk_mult=3.0)
    errs = check(prob)
    print("wide", errs)


def test_nonstandard_scale():
    prob = inputs.make_dense(B=1, N=260, Hq=2, Hkv=2, d=64, causal=False, seed=2400, scale=0.05)
    check(prob)
    prob = inputs.make_dense(B=1, N=260, Hq=2, Hkv=2, d=64, causal=True, seed=2401, scale=0.3)
    check(prob)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d,Hq,Hkv", [(128, 8, 2), (64, 4, 4)])
def test_packed_ragged_batch(d, Hq, Hkv, causal):
    lens = [5, 130, 0, 64, 257, 1, 300, 128]
    prob = inputs.make_varlen(lens, Hq=Hq, Hkv=Hkv, d=d, causal=causal, seed=2500)
    check(prob)


def test_packed_ragged_equals_dense_calls_bitwise():
    """A packed batch of equal lengths must reproduce the dense entry point bit for bit
    (every output is deterministic)."""
    prob = inputs.make_dense(B=3, N=200, Hq=4, Hkv=2, d=128, causal=True, seed=2600)
    dense = pu.run_hip(prob)
    packed = inputs.AttnProblem(name="packed", Q=prob.Q.reshape(600, 4, 128), K=prob.K.reshape(600, 2, 128),
                                V=prob.V.reshape(600, 2, 128), dO=prob.dO.reshape(600, 4, 128), Hq=4, Hkv=2, d=128,
                                scale=prob.scale, causal=True,
                                cu_seqlens=np.asarray([0, 200, 400, 600], dtype=np.int32))
    rag = pu.run_hip(packed)
    assert torch.equal(dense["O"].reshape(600, 4, 128), rag["O"])
    assert torch.equal(dense["LSE"].permute(1, 0, 2).reshape(4, 600), rag["LSE"])
    assert torch.equal(dense["dK"].reshape(600, 2, 128), rag["dK"])
    assert torch.equal(dense["dV"].reshape(600, 2, 128), rag["dV"])
    assert torch.equal(dense["dQ"].reshape(600, 4, 128), rag["dQ"])


@pytest.mark.parametrize("d", [64, 128])
def test_every_output_is_bit_reproducible(d):
    """No output is accumulated by atomic adds (dQ comes from a row-block pass of its own instead
    of section 3.2's atomic accumulation), so two runs on the same inputs agree bit for bit:
    the deterministic backward."""
    prob = inputs.make_dense(B=2, N=1333, Hq=4, Hkv=2, d=d, causal=True, seed=2700 + d)
    a = pu.run_hip(prob)
    b = pu.run_hip(prob)
    for nm in ("O", "LSE", "dQ", "dK", "dV"):
        assert torch.equal(a[nm], b[nm]), nm


def test_outputs_stay_inside_their_buffers():
    """Poisoned guard rows on both sides of every output must survive (tail blocks)."""
    from paper_2307_08691_amd import binding
    B, N, H, d, pad = 2, 130, 2, 64, 64
    prob = inputs.make_dense(B=B, N=N, Hq=H, Hkv=H, d=d, causal=True, seed=2800)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))

    def guarded(shape, dtype):
        n = int(np.prod(shape))
        buf = torch.full((n + 2 * pad * d,), float("nan"), dtype=dtype, device="cuda")
        return buf, buf[pad * d: pad * d + n].view(*shape)

    bO, O = guarded((B, N, H, d), torch.bfloat16)
    bL, L = guarded((B, H, N), torch.float32)
    binding.fa_fwd(Q, K, V, prob.scale, True, O=O, LSE=L)
    bufs = [bO, bL]
    outs = []
    for _ in range(3):
        bb, t = guarded((B, N, H, d), torch.bfloat16)
        bufs.append(bb)
        outs.append(t)
    binding.fa_bwd(Q, K, V, O, dO, L, prob.scale, True, dQ=outs[0], dK=outs[1], dV=outs[2])
    torch.cuda.synchronize()
    for bb in bufs:
        assert torch.isnan(bb[: pad * d]).all() and torch.isnan(bb[-pad * d:]).all()
    for t in [O, L] + outs:
        assert torch.isfinite(t.float()).all()


def test_closed_forms_on_the_gpu():
    """Q = 0 => O is the (prefix) mean of V and LSE = log(count); constant V => O = V."""
    prob = inputs.make_dense(B=1, N=200, Hq=2, Hkv=2, d=64, causal=True, seed=2900)
    prob.Q[...] = 0
    got = pu.run_hip(prob, backward=False)
    v = orc.widen_bf16(prob.V)[0]
    prefix = np.cumsum(v, axis=0) / np.arange(1, 201)[:, None, None]
    assert pu.maxdiff(pu.to_f64(got["O"])[0], prefix) <= 2e-2
    lse = pu.to_f64(got["LSE"])[0]
    assert pu.maxdiff(lse, np.tile(np.log(np.arange(1, 201)), (2, 1))) <= 1e-3
    prob2 = inputs.make_dense(B=1, N=200, Hq=2, Hkv=2, d=64, causal=False, seed=2901)
    prob2.V[...] = prob2.V[:, :1]
    got = pu.run_hip(prob2, backward=False)
    vv = orc.widen_bf16(prob2.V)
    assert pu.maxdiff(pu.to_f64(got["O"]), vv) <= pu.bf16_ulp(float(np.abs(vv).max()))


@pytest.mark.gpu
def test_mfma_probe_runs_and_reports_a_plausible_rate():
    """The register-resident MFMA loop: bounded by the datasheet rate at the clock it reports."""
    for rnd in (False, True):
        tf, ghz = binding.fa_mfma_probe(500, rnd)
        assert 0.5 < ghz < 2.6
        peak_at_clock = 256 * 4 * 1024 * ghz / 1e3  # TFLOP/s: 1024 FLOPs per SIMD and cycle
        assert 0.3 * peak_at_clock < tf < 1.05 * peak_at_clock


@pytest.mark.gpu
def test_forward_and_backward_replay_from_a_captured_graph():
    """The library allocates nothing and enqueues plain kernel launches on the caller's stream, so a
    whole step can be captured into a HIP graph. Replays (with other eager work and synchronisation
    in between, and new input values in the same buffers) must reproduce the eager results bit for bit."""
    import torch
    prob = inputs.make_dense(B=2, N=300, Hq=4, Hkv=2, d=128, causal=True, seed=2900)
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    B, N, Hq, d = Q.shape
    O, L = torch.empty_like(Q), torch.empty(B, Hq, N, device="cuda")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    ws = torch.empty(binding.fa_bwd_workspace_bytes(B, Hq, prob.Hkv, N, d), dtype=torch.uint8, device="cuda")

    def step():
        binding.fa_fwd(Q, K, V, prob.scale, True, O=O, LSE=L)
        binding.fa_bwd(Q, K, V, O, dO, L, prob.scale, True, dQ=dQ, dK=dK, dV=dV, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for trial in range(3):
        if trial:  # new values in the captured buffers
            Q.copy_(torch.randn_like(Q))
            dO.copy_(torch.randn_like(dO))
        step()
        torch.cuda.synchronize()
        eager = [t.clone() for t in (O, L, dQ, dK, dV)]
        for t in (O, L, dQ, dK, dV):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, (O, L, dQ, dK, dV)):
            assert torch.equal(a, b)
