"""CPU-only checks of the C ABI: the library loads, exports every function that
include/fa.h declares, and rejects bad arguments before anything is launched
(no GPU is touched: validation precedes every HIP call)."""
import ctypes
import os
import re

import pytest

from paper_2307_08691_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fa.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(fa_[a-z0-9_]+)\s*\(", src)))


def test_header_declares_the_entry_points():
    names = declared_functions()
    for must in ("fa_fwd", "fa_bwd", "fa_bwd_workspace_bytes", "fa_varlen_fwd", "fa_varlen_bwd",
                 "fa_varlen_bwd_workspace_bytes", "fa_version", "fa_status_string", "fa_last_hip_error"):
        assert must in names


def test_library_exports_every_declared_symbol_and_binding_covers_them():
    lib = binding.load()
    for name in declared_functions():
        assert hasattr(lib, name), name
        assert name in binding.SIGNATURES, name
    assert sorted(binding.SIGNATURES) == declared_functions()


def test_version_and_status_strings():
    assert binding.fa_version() >= 100
    seen = set()
    for code in range(0, -7, -1):
        s = binding.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 7
    assert binding.status_string(-99) == "unknown status"


P = 0x10000  # a non-null, 16-byte aligned fake device address; never dereferenced on these paths


def fwd(Q=P, K=P, V=P, O=P, L=P, B=1, Hq=2, Hkv=2, N=128, d=64, scale=0.125, causal=0):
    return binding.fa_fwd_raw(Q, K, V, O, L, B, Hq, Hkv, N, d, scale, causal, 0)


def bwd(ptrs=None, ws=P, ws_bytes=1 << 30, B=1, Hq=2, Hkv=2, N=128, d=64, scale=0.125, causal=0):
    ptrs = ptrs or [P] * 9
    return binding.fa_bwd_raw(*ptrs, ws, ws_bytes, B, Hq, Hkv, N, d, scale, causal, 0)


def test_fwd_rejects_bad_arguments():
    assert fwd(Q=0) == binding.FA_ERR_NULL
    assert fwd(L=0) == binding.FA_ERR_NULL
    assert fwd(B=0) == binding.FA_ERR_SHAPE
    assert fwd(N=-3) == binding.FA_ERR_SHAPE
    assert fwd(Hq=3, Hkv=2) == binding.FA_ERR_SHAPE
    assert fwd(Hkv=0) == binding.FA_ERR_SHAPE
    assert fwd(scale=0.0) == binding.FA_ERR_SHAPE
    assert fwd(scale=-1.0) == binding.FA_ERR_SHAPE
    assert fwd(scale=float("nan")) == binding.FA_ERR_SHAPE
    assert fwd(scale=float("inf")) == binding.FA_ERR_SHAPE
    assert fwd(d=100) == binding.FA_ERR_UNSUPPORTED  # not a multiple of 8
    assert fwd(d=136) == binding.FA_ERR_UNSUPPORTED
    assert fwd(d=192) == binding.FA_ERR_UNSUPPORTED  # above 128 only 256 has kernels
    assert fwd(d=264) == binding.FA_ERR_UNSUPPORTED
    assert fwd(K=P + 2) == binding.FA_ERR_ALIGN
    assert fwd(O=P + 8) == binding.FA_ERR_ALIGN


def test_bwd_rejects_bad_arguments():
    for i in range(9):
        ptrs = [P] * 9
        ptrs[i] = 0
        assert bwd(ptrs) == binding.FA_ERR_NULL
    assert bwd(ws=0) == binding.FA_ERR_NULL
    assert bwd(Hq=4, Hkv=3) == binding.FA_ERR_SHAPE
    assert bwd(d=36) == binding.FA_ERR_UNSUPPORTED
    ptrs = [P] * 9
    ptrs[6] = P + 4
    assert bwd(ptrs) == binding.FA_ERR_ALIGN
    need = binding.fa_bwd_workspace_bytes(1, 2, 2, 128, 64)
    assert bwd(ws_bytes=need - 1) == binding.FA_ERR_WORKSPACE


def test_workspace_size_formula():
    # D: one float per query row and head, rounded up to 256 bytes
    assert binding.fa_bwd_workspace_bytes(1, 2, 2, 128, 64) == 1024
    assert binding.fa_bwd_workspace_bytes(2, 16, 16, 8192, 128) == 2 * 8192 * 16 * 4
    assert binding.fa_varlen_bwd_workspace_bytes(100, 4, 2, 128) == 1792
    assert binding.fa_bwd_workspace_bytes(0, 2, 2, 128, 64) == 0
    assert binding.fa_bwd_workspace_bytes(1, 8, 2, 16, 128) >= 16 * 8 * 4


def test_varlen_rejects_bad_arguments():
    def vf(cu=P, nseq=4, total=1000, mx=400, Hq=4, Hkv=2, d=128, scale=0.1, Q=P):
        return binding.fa_varlen_fwd_raw(Q, P, P, P, P, cu, nseq, total, mx, Hq, Hkv, d, scale, 1, 0)
    assert vf(cu=0) == binding.FA_ERR_NULL
    assert vf(Q=0) == binding.FA_ERR_NULL
    assert vf(nseq=0) == binding.FA_ERR_SHAPE
    assert vf(total=0) == binding.FA_ERR_SHAPE
    assert vf(mx=2000) == binding.FA_ERR_SHAPE      # longest sequence longer than the whole batch
    assert vf(mx=100) == binding.FA_ERR_SHAPE       # 4 sequences of at most 100 cannot hold 1000 tokens
    assert vf(Hq=5) == binding.FA_ERR_SHAPE
    assert vf(d=84) == binding.FA_ERR_UNSUPPORTED

    def vb(ws_bytes=1 << 30, mx=400):
        return binding.fa_varlen_bwd_raw(*([P] * 9), P, ws_bytes, P, 4, 1000, mx, 4, 2, 128, 0.1, 1, 0)
    assert vb(ws_bytes=16) == binding.FA_ERR_WORKSPACE
    assert vb(mx=0) == binding.FA_ERR_SHAPE


def cross(Q=P, B=1, Hq=2, Hkv=2, Nq=8, Nk=128, d=64, scale=0.125, causal=0):
    return binding.fa_cross_fwd_raw(Q, P, P, P, P, B, Hq, Hkv, Nq, Nk, d, scale, causal, 0)


def test_two_length_entry_points_reject_bad_arguments():
    assert cross(Q=0) == binding.FA_ERR_NULL
    assert cross(Nq=0) == binding.FA_ERR_SHAPE
    assert cross(Nk=0) == binding.FA_ERR_SHAPE
    assert cross(Nq=129, Nk=128, causal=1) == binding.FA_ERR_SHAPE  # a query row without keys
    assert cross(d=192) == binding.FA_ERR_UNSUPPORTED
    assert cross(Q=P + 2) == binding.FA_ERR_ALIGN
    assert cross(Hq=3) == binding.FA_ERR_SHAPE
    ptrs = [P] * 9
    assert binding.fa_cross_bwd_raw(*ptrs, P, 0, 1, 2, 2, 8, 128, 64, 0.125, 0, 0) == binding.FA_ERR_WORKSPACE
    assert binding.fa_cross_bwd_raw(*ptrs, 0, 1 << 20, 1, 2, 2, 8, 128, 64, 0.125, 0, 0) == binding.FA_ERR_NULL
    # the half-precision entry points validate alike
    assert binding.fa_cross_fwd_raw(0, P, P, P, P, 1, 2, 2, 8, 128, 64, 0.125, 0, 0, f16=True) == binding.FA_ERR_NULL
    assert binding.fa_cross_fwd_raw(P, P, P, P, P, 1, 2, 2, 129, 128, 64, 0.125, 1, 0, f16=True) == binding.FA_ERR_SHAPE
    assert binding.fa_cross_bwd_raw(*ptrs, P, 0, 1, 2, 2, 8, 128, 64, 0.125, 0, 0, f16=True) == binding.FA_ERR_WORKSPACE
    # the workspace holds D: one float per query row and query head
    assert binding.fa_cross_bwd_workspace_bytes(3, 4, 2, 10, 1000, 64) == 512
    assert binding.fa_cross_bwd_workspace_bytes(3, 4, 2, 10, 1000, 64) == binding.fa_bwd_workspace_bytes(3, 4, 2, 10, 64)


def test_dropout_entry_points_reject_bad_arguments():
    def run(Q=P, p_drop=0.1, Nq=8, Nk=128, causal=0, d=64):
        return binding.fa_dropout_fwd_raw(Q, P, P, P, P, 1, 2, 2, Nq, Nk, d, 0.125, causal, p_drop, 99, 0)
    assert run(Q=0) == binding.FA_ERR_NULL
    assert run(p_drop=1.0) == binding.FA_ERR_SHAPE
    assert run(p_drop=-0.1) == binding.FA_ERR_SHAPE
    assert run(p_drop=float("nan")) == binding.FA_ERR_SHAPE
    assert run(Nq=129, causal=1) == binding.FA_ERR_SHAPE
    assert run(d=32) == binding.FA_ERR_UNSUPPORTED  # dropout: the two tile widths only
    ptrs = [P] * 9
    assert binding.fa_dropout_bwd_raw(*ptrs, P, 0, 1, 2, 2, 8, 128, 64, 0.125, 0, 0.1, 99, 0) == binding.FA_ERR_WORKSPACE
    assert binding.fa_dropout_bwd_raw(*ptrs, P, 1 << 20, 1, 2, 2, 8, 128, 64, 0.125, 0, 1.5, 99, 0) == binding.FA_ERR_SHAPE


def test_ragged_dropout_entry_points_reject_bad_arguments():
    def run(Q=P, cu=P, p_drop=0.1, d=64, mx=8):
        return binding.fa_varlen_dropout_fwd_raw(Q, P, P, P, P, cu, 2, 10, mx, 2, 2, d, 0.125, 1, p_drop, 5, 0)
    assert run(Q=0) == binding.FA_ERR_NULL
    assert run(cu=0) == binding.FA_ERR_NULL
    assert run(p_drop=1.0) == binding.FA_ERR_SHAPE
    assert run(mx=4) == binding.FA_ERR_SHAPE          # two sequences of at most 4 rows cannot hold 10
    assert run(d=96) == binding.FA_ERR_UNSUPPORTED    # dropout: the two tile widths only
    ptrs = [P] * 9
    assert binding.fa_varlen_dropout_bwd_raw(*ptrs, P, 16, P, 2, 10, 8, 2, 2, 64, 0.125, 1, 0.1, 5, 0) == binding.FA_ERR_WORKSPACE


def test_mask_entry_points_reject_bad_arguments():
    def run(Q=P, M=P, Nq=8, Nk=100, causal=0, d=64, bs=0, hs=0, rs=104):
        return binding.fa_mask_fwd_raw(Q, P, P, M, P, P, 1, 2, 2, Nq, Nk, d, 0.125, causal, bs, hs, rs, 0)
    assert run(Q=0) == binding.FA_ERR_NULL
    assert run(M=0) == binding.FA_ERR_NULL
    assert run(M=P + 8) == binding.FA_ERR_ALIGN
    assert run(rs=96) == binding.FA_ERR_SHAPE    # shorter than a row of 100 keys padded to 104
    assert run(rs=108) == binding.FA_ERR_SHAPE   # not a multiple of 8
    assert run(bs=-8) == binding.FA_ERR_SHAPE
    assert run(hs=12) == binding.FA_ERR_SHAPE
    assert run(Nq=101, causal=1) == binding.FA_ERR_SHAPE
    assert run(d=96) == binding.FA_ERR_UNSUPPORTED  # mask: the two tile widths only
    ptrs = [P] * 10
    assert binding.fa_mask_bwd_raw(*ptrs, P, 0, 1, 2, 2, 8, 100, 64, 0.125, 0, 0, 0, 104, 0) == binding.FA_ERR_WORKSPACE
    assert binding.fa_mask_bwd_raw(*ptrs, P, 1 << 20, 1, 2, 2, 8, 100, 64, 0.125, 0, 0, 0, 100, 0) == binding.FA_ERR_SHAPE


def test_ragged_two_length_entry_points_reject_bad_arguments():
    def run(Q=P, cu_q=P, cu_k=P, nseq=2, tq=10, tk=100, mq=8, mk=60, d=64):
        return binding.fa_varlen_cross_fwd_raw(Q, P, P, P, P, cu_q, cu_k, nseq, tq, tk, mq, mk, 2, 2, d, 0.125, 1, 0)
    assert run(Q=0) == binding.FA_ERR_NULL
    assert run(cu_k=0) == binding.FA_ERR_NULL
    assert run(mq=4) == binding.FA_ERR_SHAPE   # two sequences of at most 4 rows cannot hold 10
    assert run(mk=101) == binding.FA_ERR_SHAPE
    assert run(d=4) == binding.FA_ERR_UNSUPPORTED
    ptrs = [P] * 9
    assert binding.fa_varlen_cross_bwd_raw(*ptrs, P, 16, P, P, 2, 10, 100, 8, 60, 2, 2, 64, 0.125, 1, 0) == binding.FA_ERR_WORKSPACE


def test_split_key_entry_point_rejects_bad_arguments():
    def run(Q=P, ws=P, ws_bytes=1 << 30, B=1, Hq=4, Hkv=2, Nq=1, Nk=1000, d=128, scale=0.1, causal=1, splits=4):
        return binding.fa_splitkv_fwd_raw(Q, P, P, P, P, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal, splits, 0)
    assert run(Q=0) == binding.FA_ERR_NULL
    assert run(ws=0) == binding.FA_ERR_NULL
    assert run(splits=0) == binding.FA_ERR_SHAPE
    assert run(splits=129) == binding.FA_ERR_SHAPE
    assert run(Nq=1001) == binding.FA_ERR_SHAPE  # causal, more queries than keys
    assert run(ws=P + 4) == binding.FA_ERR_ALIGN
    assert run(d=256) == binding.FA_ERR_UNSUPPORTED
    assert run(d=96) == binding.FA_ERR_UNSUPPORTED  # split keys: the two tile widths only
    need = binding.fa_splitkv_fwd_workspace_bytes(1, 4, 1, 128, 4)
    assert need == 4 * 1 * 1 * 4 * 129 * 4 + (-(4 * 4 * 129 * 4)) % 256
    assert run(ws_bytes=need - 1) == binding.FA_ERR_WORKSPACE
    assert binding.splitkv_default_splits(1, 32, 8, 1, 8192) == 16
    assert binding.splitkv_default_splits(8, 32, 8, 1, 8192) == 4
    assert binding.splitkv_default_splits(64, 32, 8, 1, 8192) == 1
    assert binding.splitkv_default_splits(1, 8, 8, 1, 100) == 1
    assert binding.splitkv_default_splits(64, 32, 8, 1, 8192, ragged=True) == 1    # decode kernel: longest first
    assert binding.splitkv_default_splits(8, 32, 8, 1, 8192, ragged=True) == 4
    assert binding.splitkv_default_splits(64, 32, 8, 16, 8192, ragged=True) == 4   # 64 rows per key/value head: launch order
    assert binding.splitkv_default_splits(200, 32, 8, 1, 8192, ragged=True) == 2


def test_window_pattern_cache_fp8_and_mask_gradient_entry_points_reject_bad_arguments():
    def local(Nq=64, Nk=64, d=128, left=10, right=0, Q=P):
        return binding.fa_local_fwd_raw(Q, P, P, P, P, 1, 4, 2, Nq, Nk, d, 0.1, left, right, 0)
    assert local(Q=0) == binding.FA_ERR_NULL
    assert local(Nq=65) == binding.FA_ERR_SHAPE          # a query would stand before the first key
    assert local(d=96) == binding.FA_ERR_UNSUPPORTED     # a real window: the two tile widths only

    def vlocal(cu=P, mx=400, d=128, left=10, right=0):
        return binding.fa_varlen_local_fwd_raw(P, P, P, P, P, cu, 4, 1000, mx, 4, 2, d, 0.1, left, right, 0)
    assert vlocal(cu=0) == binding.FA_ERR_NULL
    assert vlocal(mx=2000) == binding.FA_ERR_SHAPE
    assert vlocal(d=96) == binding.FA_ERR_UNSUPPORTED

    def sparse(BM=P, block=128, bs=0, hs=0, Nk=512):
        return binding.fa_blocksparse_fwd_raw(P, P, P, BM, P, P, 1, 4, 2, 512, Nk, 128, 0.1, 0, block, bs, hs, 0)
    assert sparse(BM=0) == binding.FA_ERR_NULL
    assert sparse(block=32) == binding.FA_ERR_SHAPE      # below the kernels' key block
    assert sparse(block=96) == binding.FA_ERR_SHAPE      # not a power of two
    assert sparse(hs=-8) == binding.FA_ERR_SHAPE
    assert sparse(Nk=64 * 64 * 64 + 64) == binding.FA_ERR_UNSUPPORTED  # more key blocks than a bitmap holds

    def cache(Q=P, sl=P, table=0, page=0, pps=0, Nk=1000, d=128, splits=2, ws_bytes=1 << 30):
        return binding.fa_kvcache_fwd_raw(Q, P, P, sl, table, P, P, P, ws_bytes, 2, 4, 2, 1, Nk, d, page, pps, 0.1, 1, splits, 0)
    assert cache(Q=0) == binding.FA_ERR_NULL
    assert cache(sl=P + 2) == binding.FA_ERR_ALIGN       # lengths and tables are int32 arrays
    assert cache(table=P, page=32, pps=64) == binding.FA_ERR_UNSUPPORTED   # a page holds whole blocks of 64 keys
    assert cache(table=P, page=192, pps=8) == binding.FA_ERR_UNSUPPORTED   # and is a power of two
    assert cache(table=P, page=64, pps=15) == binding.FA_ERR_SHAPE         # 960 rows of pages for up to 1000 keys
    assert cache(table=P, page=64, pps=0) == binding.FA_ERR_SHAPE
    assert cache(d=96) == binding.FA_ERR_UNSUPPORTED
    assert cache(splits=0) == binding.FA_ERR_SHAPE
    assert cache(ws_bytes=16) == binding.FA_ERR_WORKSPACE

    def fp8(stride=1024, dq=1.0, dv=1.0, d=128, Nk=1000):
        return binding.fa_fp8_fwd_raw(P, P, P, P, P, 1, 4, 2, 64, Nk, d, stride, 0.1, dq, 1.0, dv, 0, 0)
    assert fp8(stride=1000) == binding.FA_ERR_SHAPE      # rows of V^T: a multiple of 64 bytes
    assert fp8(stride=960) == binding.FA_ERR_SHAPE       # and at least the keys rounded up to 64
    assert fp8(dq=0.0) == binding.FA_ERR_SHAPE
    assert fp8(dv=float("inf")) == binding.FA_ERR_SHAPE
    assert fp8(d=96) == binding.FA_ERR_UNSUPPORTED

    def dmask(dM=P, rs=304, hs=304 * 64, bs=304 * 64 * 4, ws_bytes=1 << 20):
        return binding.fa_mask_bwd_dmask_raw(P, P, P, P, P, P, P, P, P, P, dM, P, ws_bytes, 1, 4, 2, 64, 300, 128, 0.1, 0,
                                             0, 0, 304, bs, hs, rs, 0)
    assert dmask(dM=0) == binding.FA_ERR_NULL
    assert dmask(dM=P + 8) == binding.FA_ERR_ALIGN
    assert dmask(rs=296) == binding.FA_ERR_SHAPE         # rows shorter than the keys rounded up to 8
    assert dmask(hs=0) == binding.FA_ERR_SHAPE           # dM is never shared over heads or sequences
    assert dmask(bs=304 * 64) == binding.FA_ERR_SHAPE
    assert dmask(ws_bytes=16) == binding.FA_ERR_WORKSPACE

    # the entry point that allocates nothing: the size limit comes before anything else
    assert binding.fa_bwd_noalloc_raw(P, P, P, P, P, P, P, P, P, 64, 32, 32, 8192, 128, 0.1, 1, 0) == binding.FA_ERR_WORKSPACE


def test_mfma_probe_rejects_bad_arguments():
    assert binding.fa_mfma_probe_scratch_bytes() == 16 + 256 * 512 * 4
    assert binding.fa_mfma_probe_raw(10, 0, 0) == binding.FA_ERR_NULL
    assert binding.fa_mfma_probe_raw(10, 0, P + 8) == binding.FA_ERR_ALIGN
    assert binding.fa_mfma_probe_raw(0, 1, P) == binding.FA_ERR_SHAPE


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.load()


# ---- the tensor-level wrappers check every tensor before a pointer reaches the library

def _host(*shape, dtype=None):
    import torch
    return torch.zeros(*shape, dtype=dtype or torch.bfloat16)


def test_wrappers_reject_wrong_shapes_types_and_host_tensors_before_any_call():
    import torch
    B, N, Hq, Hkv, d = 2, 16, 4, 2, 64
    q, k = _host(B, N, Hq, d), _host(B, N, Hkv, d)
    lse = _host(B, Hq, N, dtype=torch.float32)
    cases = [
        (lambda: binding.fa_fwd(q, _host(B, N + 1, Hkv, d), k, 0.1, False), "two lengths"),
        (lambda: binding.fa_fwd(q, k, _host(B, N, Hkv, d + 8), 0.1, False), "V must have shape"),
        (lambda: binding.fa_fwd(q.float(), k, k, 0.1, False), "Q must be"),
        (lambda: binding.fa_fwd(q, k, k, 0.1, False, O=_host(B, N, Hq, d + 8)), "O must have shape"),
        (lambda: binding.fa_fwd(q, k, k, 0.1, False, LSE=_host(B, N, Hq, dtype=torch.float32)), "LSE must have shape"),
        (lambda: binding.fa_bwd(q, k, k, _host(B, N, Hkv, d), q, lse, 0.1, False), "O must have shape"),
        (lambda: binding.fa_bwd(q, k, k, q, q, lse.double(), 0.1, False), "LSE must be"),
        (lambda: binding.fa_bwd(q, k, k, q, q, lse, 0.1, False, dK=_host(B, N, Hq, d)), "dK must have shape"),
        (lambda: binding.fa_cross_bwd(q, k, k, q, q.half(), lse, 0.1, False), "dO must be"),
        (lambda: binding.fa_bwd_noalloc(q, k, k, q, q, lse, 0.1, False, None, None, None), "allocates nothing"),
        (lambda: binding.fa_varlen_fwd(_host(32, Hq, d), _host(31, Hkv, d), _host(31, Hkv, d),
                                       torch.zeros(3, dtype=torch.int32), 16, 0.1, False), "as many tokens"),
        (lambda: binding.fa_varlen_fwd(_host(32, Hq, d), _host(32, Hkv, d), _host(32, Hkv, d),
                                       torch.zeros(3, dtype=torch.int64), 16, 0.1, False), "cu_seqlens must be"),
        (lambda: binding.fa_varlen_cross_fwd(_host(32, Hq, d), _host(40, Hkv, d), _host(40, Hkv, d),
                                             torch.zeros(3, dtype=torch.int32), torch.zeros(4, dtype=torch.int32),
                                             16, 20, 0.1, False), "nseq + 1 entries each"),
        # everything right but the device: refused as well, before the library sees a pointer
        (lambda: binding.fa_fwd(q, k, k, 0.1, False), "must live on the GPU"),
        (lambda: binding.fa_bwd(q, k, k, q, q, lse, 0.1, False), "must live on the GPU"),
    ]
    for call, needle in cases:
        with pytest.raises(ValueError) as e:
            call()
        assert needle in str(e.value), (needle, str(e.value))
