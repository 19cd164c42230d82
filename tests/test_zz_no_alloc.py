"""fa_bwd_noalloc, the backward entry point that allocates nothing (its D vector lives in a static
device array inside the library), called through the C ABI: two calls in a row, the second on a
smaller problem, each bit-identical to fa_bwd on the same inputs (same kernels, and every output is
deterministic); a problem beyond the static array's size is refused before anything runs."""
import numpy as np
import pytest

from paper_2307_08691_amd import binding, inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import parity_util as pu  # noqa: E402


def both_ways(prob):
    Q, K, V, dO = (pu.to_gpu(x) for x in (prob.Q, prob.K, prob.V, prob.dO))
    O, L = binding.fa_fwd(Q, K, V, prob.scale, prob.causal)
    want = binding.fa_bwd(Q, K, V, O, dO, L, prob.scale, prob.causal)
    got = tuple(torch.full_like(t, float("nan")) for t in want)
    B, N, Hq, d = Q.shape
    torch.cuda.synchronize()
    st = binding.fa_bwd_noalloc_raw(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(), L.data_ptr(),
                                    got[0].data_ptr(), got[1].data_ptr(), got[2].data_ptr(), B, Hq, prob.Hkv, N, d,
                                    prob.scale, int(prob.causal), torch.cuda.current_stream().cuda_stream)
    assert st == binding.FA_OK, binding.status_string(st)
    torch.cuda.synchronize()
    for nm, a, b in zip(("dQ", "dK", "dV"), got, want):
        assert torch.equal(a, b), f"{prob.name}: {nm} differs from fa_bwd"
    # and the result is the right one, not merely the same one
    exp = pu.run_oracle(prob)
    ref = pu.run_reference(prob)
    pu.judge(f"fa_bwd_noalloc {pu.describe(prob)}", {nm: pu.to_f64(t) for nm, t in zip(("dQ", "dK", "dV"), got)},
             {nm: exp[nm] for nm in ("dQ", "dK", "dV")}, ref, d=prob.d)


def test_two_calls_in_a_row_the_second_smaller():
    both_ways(inputs.make_dense(B=2, N=700, Hq=4, Hkv=2, d=128, causal=True, seed=21000, name="noalloc first"))
    both_ways(inputs.make_dense(B=1, N=130, Hq=2, Hkv=2, d=64, causal=False, seed=21001, name="noalloc second"))


def test_a_problem_beyond_the_static_array_is_refused_before_anything_runs():
    q = torch.zeros(1, 16, 2, 64, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(1, 2, 16, dtype=torch.float32, device="cuda")
    out = torch.full_like(q, 7.0)
    p = q.data_ptr()
    # pointers are valid for the small shape only: the size check must come first
    rows = binding.FA_NOALLOC_MAX_ROWS
    st = binding.fa_bwd_noalloc_raw(p, p, p, p, p, lse.data_ptr(), out.data_ptr(), out.data_ptr(), out.data_ptr(),
                                    1, 2, 2, rows // 2 + 1, 64, 0.125, 0, 0)
    assert st == binding.FA_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    assert "FA_NOALLOC_MAX_ROWS" in binding.status_string(st)
