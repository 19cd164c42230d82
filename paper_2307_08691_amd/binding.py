"""Thin ctypes binding over the C ABI declared in include/fa.h.

Argument marshalling only: every step of attention runs in the HIP kernels of
libfa_gfx950.so. torch is used for device memory and the current stream. There
is no fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libfa_gfx950.so")

FA_OK = 0
FA_ERR_NULL = -1
FA_ERR_SHAPE = -2
FA_ERR_UNSUPPORTED = -3
FA_ERR_ALIGN = -4
FA_ERR_WORKSPACE = -5
FA_ERR_LAUNCH = -6

_c_int = ctypes.c_int
_c_void_p = ctypes.c_void_p
_c_float = ctypes.c_float
_c_size_t = ctypes.c_size_t

# name -> (restype, argtypes); mirrors include/fa.h one to one
SIGNATURES = {
    "fa_version": (_c_int, []),
    "fa_status_string": (ctypes.c_char_p, [_c_int]),
    "fa_last_hip_error": (_c_int, []),
    "fa_fwd": (_c_int, [_c_void_p] * 5 + [_c_int] * 5 + [_c_float, _c_int, _c_void_p]),
    "fa_bwd_workspace_bytes": (_c_size_t, [_c_int] * 5),
    "fa_bwd": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_int] * 5 + [_c_float, _c_int, _c_void_p]),
    "fa_bwd_noalloc": (_c_int, [_c_void_p] * 9 + [_c_int] * 5 + [_c_float, _c_int, _c_void_p]),
    "fa_bwd_stages": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_int] * 5 +
                      [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_varlen_fwd": (_c_int, [_c_void_p] * 5 + [_c_void_p] + [_c_int] * 6 + [_c_float, _c_int, _c_void_p]),
    "fa_varlen_fwd_f16": (_c_int, [_c_void_p] * 5 + [_c_void_p] + [_c_int] * 6 + [_c_float, _c_int, _c_void_p]),
    "fa_varlen_bwd_workspace_bytes": (_c_size_t, [_c_int] * 4),
    "fa_varlen_bwd": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_void_p] + [_c_int] * 6 +
                      [_c_float, _c_int, _c_void_p]),
    "fa_varlen_bwd_f16": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_void_p] + [_c_int] * 6 +
                      [_c_float, _c_int, _c_void_p]),
    "fa_cross_fwd": (_c_int, [_c_void_p] * 5 + [_c_int] * 6 + [_c_float, _c_int, _c_void_p]),
    "fa_cross_bwd_workspace_bytes": (_c_size_t, [_c_int] * 6),
    "fa_cross_bwd": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int, _c_void_p]),
    "fa_cross_fwd_f16": (_c_int, [_c_void_p] * 5 + [_c_int] * 6 + [_c_float, _c_int, _c_void_p]),
    "fa_cross_bwd_f16": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int, _c_void_p]),
    "fa_dropout_fwd": (_c_int, [_c_void_p] * 5 + [_c_int] * 6 + [_c_float, _c_int, _c_float, ctypes.c_uint64, _c_void_p]),
    "fa_dropout_fwd_f16": (_c_int, [_c_void_p] * 5 + [_c_int] * 6 + [_c_float, _c_int, _c_float, ctypes.c_uint64, _c_void_p]),
    "fa_dropout_bwd": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_int] * 6 +
                       [_c_float, _c_int, _c_float, ctypes.c_uint64, _c_void_p]),
    "fa_dropout_bwd_f16": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_int] * 6 +
                       [_c_float, _c_int, _c_float, ctypes.c_uint64, _c_void_p]),
    "fa_varlen_dropout_fwd": (_c_int, [_c_void_p] * 5 + [_c_void_p] + [_c_int] * 6 +
                              [_c_float, _c_int, _c_float, ctypes.c_uint64, _c_void_p]),
    "fa_varlen_dropout_fwd_f16": (_c_int, [_c_void_p] * 5 + [_c_void_p] + [_c_int] * 6 +
                              [_c_float, _c_int, _c_float, ctypes.c_uint64, _c_void_p]),
    "fa_varlen_dropout_bwd": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_void_p] + [_c_int] * 6 +
                              [_c_float, _c_int, _c_float, ctypes.c_uint64, _c_void_p]),
    "fa_varlen_dropout_bwd_f16": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_void_p] + [_c_int] * 6 +
                              [_c_float, _c_int, _c_float, ctypes.c_uint64, _c_void_p]),
    "fa_mask_fwd": (_c_int, [_c_void_p] * 6 + [_c_int] * 6 + [_c_float, _c_int] + [ctypes.c_longlong] * 3 + [_c_void_p]),
    "fa_mask_fwd_f16": (_c_int, [_c_void_p] * 6 + [_c_int] * 6 + [_c_float, _c_int] + [ctypes.c_longlong] * 3 + [_c_void_p]),
    "fa_mask_bwd": (_c_int, [_c_void_p] * 10 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int] +
                    [ctypes.c_longlong] * 3 + [_c_void_p]),
    "fa_mask_bwd_f16": (_c_int, [_c_void_p] * 10 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int] +
                    [ctypes.c_longlong] * 3 + [_c_void_p]),
    "fa_mask_bwd_dmask": (_c_int, [_c_void_p] * 11 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int] +
                          [ctypes.c_longlong] * 6 + [_c_void_p]),
    "fa_mask_bwd_dmask_f16": (_c_int, [_c_void_p] * 11 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int] +
                          [ctypes.c_longlong] * 6 + [_c_void_p]),
    "fa_local_fwd": (_c_int, [_c_void_p] * 5 + [_c_int] * 6 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_local_fwd_f16": (_c_int, [_c_void_p] * 5 + [_c_int] * 6 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_local_bwd": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_local_bwd_f16": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_varlen_local_fwd": (_c_int, [_c_void_p] * 5 + [_c_void_p] + [_c_int] * 6 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_varlen_local_fwd_f16": (_c_int, [_c_void_p] * 5 + [_c_void_p] + [_c_int] * 6 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_varlen_local_bwd": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_void_p] + [_c_int] * 6 +
                            [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_varlen_local_bwd_f16": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_void_p] + [_c_int] * 6 +
                            [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_blocksparse_fwd": (_c_int, [_c_void_p] * 6 + [_c_int] * 6 + [_c_float, _c_int, _c_int] + [ctypes.c_longlong] * 2 + [_c_void_p]),
    "fa_blocksparse_fwd_f16": (_c_int, [_c_void_p] * 6 + [_c_int] * 6 + [_c_float, _c_int, _c_int] + [ctypes.c_longlong] * 2 + [_c_void_p]),
    "fa_blocksparse_bwd": (_c_int, [_c_void_p] * 10 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int, _c_int] +
                           [ctypes.c_longlong] * 2 + [_c_void_p]),
    "fa_blocksparse_bwd_f16": (_c_int, [_c_void_p] * 10 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int, _c_int] +
                           [ctypes.c_longlong] * 2 + [_c_void_p]),
    "fa_fp8_fwd": (_c_int, [_c_void_p] * 5 + [_c_int] * 6 + [ctypes.c_longlong] + [_c_float] * 4 + [_c_int, _c_void_p]),
    "fa_varlen_cross_fwd": (_c_int, [_c_void_p] * 5 + [_c_void_p] * 2 + [_c_int] * 8 + [_c_float, _c_int, _c_void_p]),
    "fa_varlen_cross_fwd_f16": (_c_int, [_c_void_p] * 5 + [_c_void_p] * 2 + [_c_int] * 8 + [_c_float, _c_int, _c_void_p]),
    "fa_varlen_cross_bwd": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_void_p] * 2 + [_c_int] * 8 +
                            [_c_float, _c_int, _c_void_p]),
    "fa_varlen_cross_bwd_f16": (_c_int, [_c_void_p] * 9 + [_c_void_p, _c_size_t] + [_c_void_p] * 2 + [_c_int] * 8 +
                            [_c_float, _c_int, _c_void_p]),
    "fa_splitkv_fwd_workspace_bytes": (_c_size_t, [_c_int] * 5),
    "fa_splitkv_fwd": (_c_int, [_c_void_p] * 5 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_splitkv_fwd_f16": (_c_int, [_c_void_p] * 5 + [_c_void_p, _c_size_t] + [_c_int] * 6 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_kvcache_fwd": (_c_int, [_c_void_p] * 7 + [_c_void_p, _c_size_t] + [_c_int] * 8 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_kvcache_fwd_f16": (_c_int, [_c_void_p] * 7 + [_c_void_p, _c_size_t] + [_c_int] * 8 + [_c_float, _c_int, _c_int, _c_void_p]),
    "fa_mfma_probe_scratch_bytes": (_c_size_t, []),
    "fa_mfma_probe": (_c_int, [_c_int, _c_int, _c_void_p, _c_void_p]),
}

_lib = None


class FaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"fa status {status}: {message}")
        self.status = status


def load() -> ctypes.CDLL:
    """Load the shared library (once). Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2307_08691_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().fa_status_string(status).decode()


def _check(status: int) -> None:
    if status != FA_OK:
        raise FaError(status, status_string(status))


def _ptr(t) -> int:
    """Device address of a tensor for the C ABI (None -> NULL). Host tensors stop here."""
    if t is None:
        return 0
    if not t.is_cuda:
        raise ValueError("every tensor must live on the GPU")
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def fa_version() -> int:
    return load().fa_version()


# ---------------------------------------------------------------------------
# raw calls: pointers and sizes in, status out (used by the error-path tests)
# ---------------------------------------------------------------------------

def fa_fwd_raw(Q, K, V, O, LSE, B, Hq, Hkv, N, d, scale, causal, stream=0) -> int:
    return load().fa_fwd(Q, K, V, O, LSE, B, Hq, Hkv, N, d, scale, int(causal), stream)


def fa_bwd_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, N, d, scale, causal, stream=0) -> int:
    return load().fa_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, N, d, scale, int(causal), stream)


def fa_bwd_noalloc_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, B, Hq, Hkv, N, d, scale, causal, stream=0) -> int:
    return load().fa_bwd_noalloc(Q, K, V, O, dO, LSE, dQ, dK, dV, B, Hq, Hkv, N, d, scale, int(causal), stream)


def fa_bwd_stages_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, N, d, scale, causal, stages,
                      stream=0) -> int:
    return load().fa_bwd_stages(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, N, d, scale, int(causal),
                                stages, stream)


def fa_varlen_fwd_raw(Q, K, V, O, LSE, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale, causal, stream=0, f16=False) -> int:
    fn = load().fa_varlen_fwd_f16 if f16 else load().fa_varlen_fwd
    return fn(Q, K, V, O, LSE, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale, int(causal), stream)


def fa_varlen_bwd_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale,
                      causal, stream=0, f16=False) -> int:
    fn = load().fa_varlen_bwd_f16 if f16 else load().fa_varlen_bwd
    return fn(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale,
              int(causal), stream)


def fa_bwd_workspace_bytes(B, Hq, Hkv, N, d) -> int:
    return load().fa_bwd_workspace_bytes(B, Hq, Hkv, N, d)


def fa_varlen_bwd_workspace_bytes(total, Hq, Hkv, d) -> int:
    return load().fa_varlen_bwd_workspace_bytes(total, Hq, Hkv, d)


def fa_cross_fwd_raw(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, stream=0, f16=False) -> int:
    fn = load().fa_cross_fwd_f16 if f16 else load().fa_cross_fwd
    return fn(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), stream)


def fa_cross_bwd_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal,
                     stream=0, f16=False) -> int:
    fn = load().fa_cross_bwd_f16 if f16 else load().fa_cross_bwd
    return fn(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), stream)


def fa_cross_bwd_workspace_bytes(B, Hq, Hkv, Nq, Nk, d) -> int:
    return load().fa_cross_bwd_workspace_bytes(B, Hq, Hkv, Nq, Nk, d)


def fa_dropout_fwd_raw(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, p_drop, seed, stream=0, f16=False) -> int:
    fn = load().fa_dropout_fwd_f16 if f16 else load().fa_dropout_fwd
    return fn(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), p_drop, seed, stream)


def fa_dropout_bwd_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal, p_drop,
                       seed, stream=0, f16=False) -> int:
    fn = load().fa_dropout_bwd_f16 if f16 else load().fa_dropout_bwd
    return fn(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), p_drop, seed,
              stream)


def fa_varlen_dropout_fwd_raw(Q, K, V, O, LSE, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale, causal, p_drop, seed,
                              stream=0, f16=False) -> int:
    fn = load().fa_varlen_dropout_fwd_f16 if f16 else load().fa_varlen_dropout_fwd
    return fn(Q, K, V, O, LSE, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale, int(causal), p_drop, seed, stream)


def fa_varlen_dropout_bwd_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, cu, nseq, total, max_seqlen, Hq, Hkv, d,
                              scale, causal, p_drop, seed, stream=0, f16=False) -> int:
    fn = load().fa_varlen_dropout_bwd_f16 if f16 else load().fa_varlen_dropout_bwd
    return fn(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale,
              int(causal), p_drop, seed, stream)


def fa_mask_fwd_raw(Q, K, V, M, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, mask_bs, mask_hs, mask_rs, stream=0, f16=False) -> int:
    fn = load().fa_mask_fwd_f16 if f16 else load().fa_mask_fwd
    return fn(Q, K, V, M, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), mask_bs, mask_hs, mask_rs, stream)


def fa_mask_bwd_raw(Q, K, V, M, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal, mask_bs,
                    mask_hs, mask_rs, stream=0, f16=False) -> int:
    fn = load().fa_mask_bwd_f16 if f16 else load().fa_mask_bwd
    return fn(Q, K, V, M, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), mask_bs,
              mask_hs, mask_rs, stream)


def fa_mask_bwd_dmask_raw(Q, K, V, M, O, dO, LSE, dQ, dK, dV, dM, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal, mask_bs,
                          mask_hs, mask_rs, dm_bs, dm_hs, dm_rs, stream=0, f16=False) -> int:
    fn = load().fa_mask_bwd_dmask_f16 if f16 else load().fa_mask_bwd_dmask
    return fn(Q, K, V, M, O, dO, LSE, dQ, dK, dV, dM, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), mask_bs,
              mask_hs, mask_rs, dm_bs, dm_hs, dm_rs, stream)


def fa_local_fwd_raw(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, left, right, stream=0, f16=False) -> int:
    fn = load().fa_local_fwd_f16 if f16 else load().fa_local_fwd
    return fn(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, left, right, stream)


def fa_local_bwd_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, left, right, stream=0, f16=False) -> int:
    fn = load().fa_local_bwd_f16 if f16 else load().fa_local_bwd
    return fn(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, left, right, stream)


def fa_varlen_local_fwd_raw(Q, K, V, O, LSE, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale, left, right, stream=0, f16=False) -> int:
    fn = load().fa_varlen_local_fwd_f16 if f16 else load().fa_varlen_local_fwd
    return fn(Q, K, V, O, LSE, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale, left, right, stream)


def fa_varlen_local_bwd_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale,
                            left, right, stream=0, f16=False) -> int:
    fn = load().fa_varlen_local_bwd_f16 if f16 else load().fa_varlen_local_bwd
    return fn(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, cu, nseq, total, max_seqlen, Hq, Hkv, d, scale, left,
              right, stream)


def fa_blocksparse_fwd_raw(Q, K, V, BM, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, block, bs, hs, stream=0, f16=False) -> int:
    fn = load().fa_blocksparse_fwd_f16 if f16 else load().fa_blocksparse_fwd
    return fn(Q, K, V, BM, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), block, bs, hs, stream)


def fa_blocksparse_bwd_raw(Q, K, V, BM, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal, block,
                           bs, hs, stream=0, f16=False) -> int:
    fn = load().fa_blocksparse_bwd_f16 if f16 else load().fa_blocksparse_bwd
    return fn(Q, K, V, BM, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), block, bs,
              hs, stream)


def fa_fp8_fwd_raw(Q8, K8, Vt8, O, LSE, B, Hq, Hkv, Nq, Nk, d, vt_stride, scale, dq, dk, dv, causal, stream=0) -> int:
    return load().fa_fp8_fwd(Q8, K8, Vt8, O, LSE, B, Hq, Hkv, Nq, Nk, d, vt_stride, scale, dq, dk, dv, int(causal), stream)


def fa_varlen_cross_fwd_raw(Q, K, V, O, LSE, cu_q, cu_k, nseq, total_q, total_k, max_q, max_k, Hq, Hkv, d, scale,
                            causal, stream=0, f16=False) -> int:
    fn = load().fa_varlen_cross_fwd_f16 if f16 else load().fa_varlen_cross_fwd
    return fn(Q, K, V, O, LSE, cu_q, cu_k, nseq, total_q, total_k, max_q, max_k, Hq, Hkv, d, scale, int(causal),
              stream)


def fa_varlen_cross_bwd_raw(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, cu_q, cu_k, nseq, total_q, total_k, max_q,
                            max_k, Hq, Hkv, d, scale, causal, stream=0, f16=False) -> int:
    fn = load().fa_varlen_cross_bwd_f16 if f16 else load().fa_varlen_cross_bwd
    return fn(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ws_bytes, cu_q, cu_k, nseq, total_q, total_k, max_q, max_k, Hq,
              Hkv, d, scale, int(causal), stream)


def fa_splitkv_fwd_workspace_bytes(B, Hq, Nq, d, num_splits) -> int:
    return load().fa_splitkv_fwd_workspace_bytes(B, Hq, Nq, d, num_splits)


def fa_splitkv_fwd_raw(Q, K, V, O, LSE, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal, num_splits, stream=0, f16=False) -> int:
    fn = load().fa_splitkv_fwd_f16 if f16 else load().fa_splitkv_fwd
    return fn(Q, K, V, O, LSE, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, scale, int(causal), num_splits, stream)


def fa_kvcache_fwd_raw(Q, Kc, Vc, seqlens_k, block_table, O, LSE, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, page_size,
                       pages_per_seq, scale, causal, num_splits, stream=0, f16=False) -> int:
    fn = load().fa_kvcache_fwd_f16 if f16 else load().fa_kvcache_fwd
    return fn(Q, Kc, Vc, seqlens_k, block_table, O, LSE, ws, ws_bytes, B, Hq, Hkv, Nq, Nk, d, page_size,
              pages_per_seq, scale, int(causal), num_splits, stream)


def fa_mfma_probe_scratch_bytes() -> int:
    return load().fa_mfma_probe_scratch_bytes()


def fa_mfma_probe_raw(iters, random_operands, scratch, stream=0) -> int:
    return load().fa_mfma_probe(iters, int(random_operands), scratch, stream)


# ---------------------------------------------------------------------------
# tensor-level wrappers: same names as the C entry points
#
# The C ABI sees raw pointers and sizes; a tensor of the wrong shape, type or device would become
# an out-of-bounds device access there. Every tensor is therefore checked here, before the call:
# device, contiguity, element type and the exact shape its role implies.
# ---------------------------------------------------------------------------

def _need(t, name, dtype=None, shape=None, device=None):
    # (type and shape first, so that these checks can be exercised with host tensors)
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, not {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, not {tuple(t.shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if device is not None and t.device != device:
        raise ValueError(f"{name} must be on {device}, like Q")
    # (that the common device is a GPU is checked where the pointers are taken, in _ptr)


def _elem_type(Q, allowed=None):
    import torch
    allowed = allowed or (torch.bfloat16, torch.float16)
    if Q.dtype not in allowed:
        raise ValueError("Q must be " + " or ".join(str(a) for a in allowed))
    return Q.dtype


def _out(t, name, shape, dtype, device):
    """An output tensor: allocated when the caller passed none, checked otherwise."""
    import torch
    if t is None:
        return torch.empty(tuple(shape), dtype=dtype, device=device)
    _need(t, name, dtype, shape, device)
    return t


def _workspace(ws, nbytes, device):
    import torch
    if ws is None:
        return torch.empty(nbytes, dtype=torch.uint8, device=device)
    _need(ws, "workspace", None, None, device)
    if ws.numel() * ws.element_size() < nbytes:
        raise ValueError(f"workspace holds {ws.numel() * ws.element_size()} bytes, {nbytes} are needed")
    return ws


def _wsbytes(ws) -> int:
    return ws.numel() * ws.element_size()


class _Dims:
    pass


def _dense(Q, K, V, allowed=None, one_length=False):
    """Q [B,Nq,Hq,d], K, V [B,Nk,Hkv,d] of one element type on one device -> their dimensions."""
    et = _elem_type(Q, allowed)
    _need(Q, "Q", et)
    if Q.dim() != 4 or K.dim() != 4:
        raise ValueError("Q must be [B, Nq, Hq, d] and K, V [B, Nk, Hkv, d]")
    x = _Dims()
    x.B, x.Nq, x.Hq, x.d = Q.shape
    x.Nk, x.Hkv = K.shape[1], K.shape[2]
    x.et, x.dev = et, Q.device
    if one_length and x.Nk != x.Nq:
        raise ValueError("K, V must be [B, N, Hkv, d] with the N of Q (two lengths: the fa_cross_* entry points)")
    _need(K, "K", et, (x.B, x.Nk, x.Hkv, x.d), x.dev)
    _need(V, "V", et, (x.B, x.Nk, x.Hkv, x.d), x.dev)
    x.q_shape, x.k_shape, x.l_shape = (x.B, x.Nq, x.Hq, x.d), (x.B, x.Nk, x.Hkv, x.d), (x.B, x.Hq, x.Nq)
    return x


def _packed(Q, K, V, cu_q, cu_k=None, allowed=None):
    """Q [Tq,Hq,d], K, V [Tk,Hkv,d] of one element type (bf16 unless `allowed` says otherwise) and the
    int32 offset arrays (one for one length) -> dimensions."""
    import torch
    et = _elem_type(Q, allowed or (torch.bfloat16,))
    _need(Q, "Q", et)
    if Q.dim() != 3 or K.dim() != 3:
        raise ValueError("Q must be [T, Hq, d] and K, V [T, Hkv, d]")
    x = _Dims()
    x.Tq, x.Hq, x.d = Q.shape
    x.Tk, x.Hkv = K.shape[0], K.shape[1]
    x.et, x.dev = et, Q.device
    if cu_k is None and x.Tk != x.Tq:
        raise ValueError("K, V must hold as many tokens as Q (two lengths: the fa_varlen_cross_* entry points)")
    _need(K, "K", x.et, (x.Tk, x.Hkv, x.d), x.dev)
    _need(V, "V", x.et, (x.Tk, x.Hkv, x.d), x.dev)
    for t, nm in ((cu_q, "cu_seqlens"), (cu_k, "cu_seqlens_k")):
        if t is not None:
            _need(t, nm, torch.int32, None, x.dev)
            if t.dim() != 1 or t.numel() < 2:
                raise ValueError(f"{nm} must be a vector of nseq + 1 offsets")
    x.nseq = cu_q.numel() - 1
    if cu_k is not None and cu_k.numel() != cu_q.numel():
        raise ValueError("the two offset arrays must have nseq + 1 entries each")
    x.q_shape, x.k_shape, x.l_shape = (x.Tq, x.Hq, x.d), (x.Tk, x.Hkv, x.d), (x.Hq, x.Tq)
    return x


def _fwd_outputs(x, O, LSE):
    import torch
    return _out(O, "O", x.q_shape, x.et, x.dev), _out(LSE, "LSE", x.l_shape, torch.float32, x.dev)


def _bwd_tensors(x, O, dO, LSE, dQ, dK, dV):
    import torch
    _need(O, "O", x.et, x.q_shape, x.dev)
    _need(dO, "dO", x.et, x.q_shape, x.dev)
    _need(LSE, "LSE", torch.float32, x.l_shape, x.dev)
    return (_out(dQ, "dQ", x.q_shape, x.et, x.dev), _out(dK, "dK", x.k_shape, x.et, x.dev),
            _out(dV, "dV", x.k_shape, x.et, x.dev))


def fa_fwd(Q, K, V, scale: float, causal: bool, O=None, LSE=None) -> Tuple["torch.Tensor", "torch.Tensor"]:
    """Dense forward. Q [B,N,Hq,d], K,V [B,N,Hkv,d] bf16 -> O [B,N,Hq,d] bf16, LSE [B,Hq,N] fp32."""
    import torch
    x = _dense(Q, K, V, (torch.bfloat16,), one_length=True)
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), x.B, x.Hq, x.Hkv, x.Nq, x.d, scale, causal, _stream()))
    return O, LSE


def fa_bwd(Q, K, V, O, dO, LSE, scale: float, causal: bool, dQ=None, dK=None, dV=None, workspace=None):
    """Dense backward. Returns dQ [B,N,Hq,d], dK, dV [B,N,Hkv,d] (bf16)."""
    import torch
    x = _dense(Q, K, V, (torch.bfloat16,), one_length=True)
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_bwd_workspace_bytes(x.B, x.Hq, x.Hkv, x.Nq, x.d), x.dev)
    _check(fa_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK), _ptr(dV),
                      _ptr(ws), _wsbytes(ws), x.B, x.Hq, x.Hkv, x.Nq, x.d, scale, causal, _stream()))
    return dQ, dK, dV


FA_NOALLOC_MAX_ROWS = 2 * 1024 * 1024  # (query row, head) pairs that fa_bwd_noalloc's static scratch holds


def fa_bwd_noalloc(Q, K, V, O, dO, LSE, scale: float, causal: bool, dQ, dK, dV) -> None:
    """Dense backward into caller-supplied dQ, dK, dV without a workspace: nothing is allocated,
    here or in the library (D lives in a static device array; at most FA_NOALLOC_MAX_ROWS
    (query row, head) pairs). Calls on one GPU must not overlap."""
    import torch
    x = _dense(Q, K, V, (torch.bfloat16,), one_length=True)
    if dQ is None or dK is None or dV is None:
        raise ValueError("fa_bwd_noalloc allocates nothing: pass dQ, dK and dV")
    _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    _check(fa_bwd_noalloc_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK), _ptr(dV),
                              x.B, x.Hq, x.Hkv, x.Nq, x.d, scale, causal, _stream()))


def fa_bwd_stages(Q, K, V, O, dO, LSE, scale: float, causal: bool, stages: int, dQ, dK, dV, workspace) -> None:
    """Profiling aid: run the selected stages (1 D pre-pass | 2 dK/dV | 4 dQ) of the dense backward."""
    import torch
    x = _dense(Q, K, V, (torch.bfloat16,), one_length=True)
    _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_bwd_workspace_bytes(x.B, x.Hq, x.Hkv, x.Nq, x.d), x.dev)
    _check(fa_bwd_stages_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK), _ptr(dV),
                             _ptr(ws), _wsbytes(ws), x.B, x.Hq, x.Hkv, x.Nq, x.d, scale, causal, stages, _stream()))


def fa_varlen_fwd(Q, K, V, cu_seqlens, max_seqlen: int, scale: float, causal: bool, O=None, LSE=None):
    """Packed ragged forward. Q [T,Hq,d], K,V [T,Hkv,d] bf16, cu_seqlens int32 on the GPU.
    Returns O [T,Hq,d] bf16 and LSE [Hq,T] fp32."""
    import torch
    x = _packed(Q, K, V, cu_seqlens, allowed=(torch.bfloat16, torch.float16))
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_varlen_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(cu_seqlens), x.nseq, x.Tq, max_seqlen,
                             x.Hq, x.Hkv, x.d, scale, causal, _stream(), x.et == torch.float16))
    return O, LSE


def fa_varlen_bwd(Q, K, V, O, dO, LSE, cu_seqlens, max_seqlen: int, scale: float, causal: bool,
                  dQ=None, dK=None, dV=None, workspace=None):
    """Packed ragged backward. Returns dQ [T,Hq,d], dK, dV [T,Hkv,d] (bf16)."""
    import torch
    x = _packed(Q, K, V, cu_seqlens, allowed=(torch.bfloat16, torch.float16))
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_varlen_bwd_workspace_bytes(x.Tq, x.Hq, x.Hkv, x.d), x.dev)
    _check(fa_varlen_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK), _ptr(dV),
                             _ptr(ws), _wsbytes(ws), _ptr(cu_seqlens), x.nseq, x.Tq, max_seqlen, x.Hq, x.Hkv, x.d, scale,
                             causal, _stream(), x.et == torch.float16))
    return dQ, dK, dV


def fa_cross_fwd(Q, K, V, scale: float, causal: bool, O=None, LSE=None):
    """Two lengths. Q [B,Nq,Hq,d], K,V [B,Nk,Hkv,d] bf16 (fa_cross_fwd) or fp16 (fa_cross_fwd_f16)
    -> O [B,Nq,Hq,d] of the same type, LSE [B,Hq,Nq] fp32."""
    import torch
    x = _dense(Q, K, V)
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_cross_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, scale, causal,
                            _stream(), x.et == torch.float16))
    return O, LSE


def fa_cross_bwd(Q, K, V, O, dO, LSE, scale: float, causal: bool, dQ=None, dK=None, dV=None, workspace=None):
    """Two lengths, backward (bf16 or fp16 by the tensors' type). Returns dQ [B,Nq,Hq,d], dK, dV [B,Nk,Hkv,d]."""
    import torch
    x = _dense(Q, K, V)
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_cross_bwd_workspace_bytes(x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d), x.dev)
    _check(fa_cross_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK), _ptr(dV),
                            _ptr(ws), _wsbytes(ws), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, scale, causal, _stream(),
                            x.et == torch.float16))
    return dQ, dK, dV


def fa_dropout_fwd(Q, K, V, scale: float, causal: bool, p_drop: float, seed: int, O=None, LSE=None):
    """Forward with dropout on P. Q [B,Nq,Hq,d], K,V [B,Nk,Hkv,d] bf16 or fp16."""
    import torch
    x = _dense(Q, K, V)
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_dropout_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, scale,
                              causal, p_drop, seed, _stream(), x.et == torch.float16))
    return O, LSE


def fa_dropout_bwd(Q, K, V, O, dO, LSE, scale: float, causal: bool, p_drop: float, seed: int, dQ=None, dK=None,
                   dV=None, workspace=None):
    """Backward with the dropout mask of fa_dropout_fwd for the same p_drop and seed."""
    import torch
    x = _dense(Q, K, V)
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_cross_bwd_workspace_bytes(x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d), x.dev)
    _check(fa_dropout_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK), _ptr(dV),
                              _ptr(ws), _wsbytes(ws), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, scale, causal, p_drop, seed,
                              _stream(), x.et == torch.float16))
    return dQ, dK, dV


def fa_varlen_dropout_fwd(Q, K, V, cu_seqlens, max_seqlen: int, scale: float, causal: bool, p_drop: float, seed: int,
                          O=None, LSE=None):
    """Packed ragged forward with dropout on P. Q [T,Hq,d], K,V [T,Hkv,d] bf16; cu_seqlens int32 on the GPU."""
    import torch
    x = _packed(Q, K, V, cu_seqlens, allowed=(torch.bfloat16, torch.float16))
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_varlen_dropout_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(cu_seqlens), x.nseq, x.Tq,
                                     max_seqlen, x.Hq, x.Hkv, x.d, scale, causal, p_drop, seed, _stream(), x.et == torch.float16))
    return O, LSE


def fa_varlen_dropout_bwd(Q, K, V, O, dO, LSE, cu_seqlens, max_seqlen: int, scale: float, causal: bool, p_drop: float,
                          seed: int, dQ=None, dK=None, dV=None, workspace=None):
    """Packed ragged backward with the dropout mask of fa_varlen_dropout_fwd for the same p_drop and seed."""
    import torch
    x = _packed(Q, K, V, cu_seqlens, allowed=(torch.bfloat16, torch.float16))
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_varlen_bwd_workspace_bytes(x.Tq, x.Hq, x.Hkv, x.d), x.dev)
    _check(fa_varlen_dropout_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK),
                                     _ptr(dV), _ptr(ws), _wsbytes(ws), _ptr(cu_seqlens), x.nseq, x.Tq, max_seqlen, x.Hq,
                                     x.Hkv, x.d, scale, causal, p_drop, seed, _stream(), x.et == torch.float16))
    return dQ, dK, dV


def mask_buffer(Bm: int, Hm: int, Nq: int, Nk: int, device="cuda", dtype=None):
    """An elementwise mask [Bm, Hm, Nq, Nk] (zeros; bf16, or the fp16 of fp16 Q, K, V) whose rows are
    padded in memory to a multiple of 8 elements, as fa_mask_fwd / fa_mask_bwd require; Bm, Hm = 1
    shares the mask."""
    import torch
    rs = (Nk + 7) // 8 * 8
    return torch.zeros((Bm, Hm, Nq, rs), dtype=dtype or torch.bfloat16, device=device)[..., :Nk]


def _mask_strides(M, x):
    import torch
    if M.dtype != x.et or M.device != x.dev:
        raise ValueError("M must have the element type of Q and live on its device")
    if M.dim() != 4 or M.shape[0] not in (1, x.B) or M.shape[1] not in (1, x.Hq) or tuple(M.shape[2:]) != (x.Nq, x.Nk):
        raise ValueError("M must be [1 or B, 1 or Hq, Nq, Nk]")
    if M.stride(3) != 1:
        raise ValueError("the key dimension of M must be contiguous")
    return (M.stride(0) if M.shape[0] > 1 else 0, M.stride(1) if M.shape[1] > 1 else 0, M.stride(2))


def fa_mask_fwd(Q, K, V, M, scale: float, causal: bool, O=None, LSE=None):
    """Forward with the mask M added to the scaled scores. Q [B,Nq,Hq,d], K,V [B,Nk,Hkv,d] bf16 or fp16; M (same type) as
    made by mask_buffer (entries finite or -inf)."""
    import torch
    x = _dense(Q, K, V)
    bs, hs, rs = _mask_strides(M, x)
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_mask_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(M), _ptr(O), _ptr(LSE), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d,
                           scale, causal, bs, hs, rs, _stream(), x.et == torch.float16))
    return O, LSE


def fa_mask_bwd(Q, K, V, M, O, dO, LSE, scale: float, causal: bool, dQ=None, dK=None, dV=None, workspace=None):
    """Backward with the mask of fa_mask_fwd; M receives no gradient."""
    import torch
    x = _dense(Q, K, V)
    bs, hs, rs = _mask_strides(M, x)
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_cross_bwd_workspace_bytes(x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d), x.dev)
    _check(fa_mask_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(M), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK),
                           _ptr(dV), _ptr(ws), _wsbytes(ws), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, scale, causal, bs, hs, rs,
                           _stream(), x.et == torch.float16))
    return dQ, dK, dV


def fa_mask_bwd_dmask(Q, K, V, M, O, dO, LSE, scale: float, causal: bool, dQ=None, dK=None, dV=None, dM=None, workspace=None):
    """fa_mask_bwd that also returns dM [B, Hq, Nq, Nk] (the gradient of a mask read as a bias), a view
    into a zero-filled buffer whose rows are padded to a multiple of 8 elements. A caller-supplied dM
    must be such a view (mask_buffer(B, Hq, Nq, Nk, dtype=...)) and, under the causal rule, zero-filled."""
    import torch
    x = _dense(Q, K, V)
    bs, hs, rs = _mask_strides(M, x)
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    if dM is None:
        dM = mask_buffer(x.B, x.Hq, x.Nq, x.Nk, device=x.dev, dtype=x.et)
    if dM.dtype != x.et or dM.device != x.dev or tuple(dM.shape) != (x.B, x.Hq, x.Nq, x.Nk) or dM.stride(3) != 1:
        raise ValueError("dM must be [B, Hq, Nq, Nk] of the element type of Q, on its device, key dimension contiguous")
    ws = _workspace(workspace, fa_cross_bwd_workspace_bytes(x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d), x.dev)
    _check(fa_mask_bwd_dmask_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(M), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK),
                                 _ptr(dV), _ptr(dM), _ptr(ws), _wsbytes(ws), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, scale,
                                 causal, bs, hs, rs, dM.stride(0), dM.stride(1), dM.stride(2), _stream(),
                                 x.et == torch.float16))
    return dQ, dK, dV, dM


def fa_local_fwd(Q, K, V, scale: float, window_left: int, window_right: int, O=None, LSE=None):
    """Sliding window: the query at position q = r + Nk - Nq sees keys q - window_left .. q + window_right
    (a negative bound: none). Q [B,Nq,Hq,d], K,V [B,Nk,Hkv,d] bf16 or fp16."""
    import torch
    x = _dense(Q, K, V)
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_local_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, scale,
                            window_left, window_right, _stream(), x.et == torch.float16))
    return O, LSE


def fa_local_bwd(Q, K, V, O, dO, LSE, scale: float, window_left: int, window_right: int, dQ=None, dK=None, dV=None,
                 workspace=None):
    """Backward of fa_local_fwd for the same window."""
    import torch
    x = _dense(Q, K, V)
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_cross_bwd_workspace_bytes(x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d), x.dev)
    _check(fa_local_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK), _ptr(dV),
                            _ptr(ws), _wsbytes(ws), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, scale, window_left, window_right,
                            _stream(), x.et == torch.float16))
    return dQ, dK, dV


def fa_varlen_local_fwd(Q, K, V, cu_seqlens, max_seqlen: int, scale: float, window_left: int, window_right: int,
                        O=None, LSE=None):
    """Packed ragged forward with the sliding window of fa_local_fwd inside every sequence. Q [T,Hq,d],
    K,V [T,Hkv,d] bf16; cu_seqlens int32 on the GPU."""
    import torch
    x = _packed(Q, K, V, cu_seqlens, allowed=(torch.bfloat16, torch.float16))
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_varlen_local_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(cu_seqlens), x.nseq, x.Tq,
                                   max_seqlen, x.Hq, x.Hkv, x.d, scale, window_left, window_right, _stream(), x.et == torch.float16))
    return O, LSE


def fa_varlen_local_bwd(Q, K, V, O, dO, LSE, cu_seqlens, max_seqlen: int, scale: float, window_left: int,
                        window_right: int, dQ=None, dK=None, dV=None, workspace=None):
    """Backward of fa_varlen_local_fwd for the same window."""
    import torch
    x = _packed(Q, K, V, cu_seqlens, allowed=(torch.bfloat16, torch.float16))
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_varlen_bwd_workspace_bytes(x.Tq, x.Hq, x.Hkv, x.d), x.dev)
    _check(fa_varlen_local_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK),
                                   _ptr(dV), _ptr(ws), _wsbytes(ws), _ptr(cu_seqlens), x.nseq, x.Tq, max_seqlen, x.Hq,
                                   x.Hkv, x.d, scale, window_left, window_right, _stream(), x.et == torch.float16))
    return dQ, dK, dV


def _block_mask_strides(BM, x, block):
    import torch
    nrb, ncb = -(-x.Nq // block), -(-x.Nk // block)
    if BM.dtype != torch.uint8 or BM.device != x.dev or not BM.is_contiguous():
        raise ValueError("block_mask must be a contiguous uint8 tensor on the device of Q")
    if BM.dim() != 4 or BM.shape[0] not in (1, x.B) or BM.shape[1] not in (1, x.Hq) or tuple(BM.shape[2:]) != (nrb, ncb):
        raise ValueError(f"block_mask must be [1 or B, 1 or Hq, {nrb}, {ncb}]")
    return (BM.stride(0) if BM.shape[0] > 1 else 0, BM.stride(1) if BM.shape[1] > 1 else 0)


def fa_blocksparse_fwd(Q, K, V, block_mask, block: int, scale: float, causal: bool, O=None, LSE=None):
    """Block-sparse forward: block_mask uint8 [1 or B, 1 or Hq, ceil(Nq/block), ceil(Nk/block)], non-zero = the
    block of `block` x `block` scores takes part. Q [B,Nq,Hq,d], K,V [B,Nk,Hkv,d] bf16 or fp16."""
    import torch
    x = _dense(Q, K, V)
    bs, hs = _block_mask_strides(block_mask, x, block)
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_blocksparse_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(block_mask), _ptr(O), _ptr(LSE), x.B, x.Hq, x.Hkv, x.Nq,
                                  x.Nk, x.d, scale, causal, block, bs, hs, _stream(), x.et == torch.float16))
    return O, LSE


def fa_blocksparse_bwd(Q, K, V, block_mask, block: int, O, dO, LSE, scale: float, causal: bool, dQ=None, dK=None, dV=None,
                       workspace=None):
    """Backward of fa_blocksparse_fwd for the same pattern."""
    import torch
    x = _dense(Q, K, V)
    bs, hs = _block_mask_strides(block_mask, x, block)
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_cross_bwd_workspace_bytes(x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d), x.dev)
    _check(fa_blocksparse_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(block_mask), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ),
                                  _ptr(dK), _ptr(dV), _ptr(ws), _wsbytes(ws), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, scale,
                                  causal, block, bs, hs, _stream(), x.et == torch.float16))
    return dQ, dK, dV


def fp8_key_major(V8):
    """V8 [B, Nk, Hkv, d] uint8 (E4M3 bytes) -> the key-major tensor fa_fp8_fwd takes: [B, Hkv, d, stride] with
    stride = Nk rounded up to 64, the padding zero."""
    import torch
    B, Nk, Hkv, d = V8.shape
    stride = (Nk + 63) // 64 * 64
    Vt = torch.zeros((B, Hkv, d, stride), dtype=torch.uint8, device=V8.device)
    Vt[..., :Nk] = V8.permute(0, 2, 3, 1)
    return Vt


def fa_fp8_fwd(Q8, K8, Vt8, Nk: int, scale: float, descale_q: float, descale_k: float, descale_v: float, causal: bool,
               O=None, LSE=None):
    """Forward on E4M3 operands. Q8 [B,Nq,Hq,d], K8 [B,Nk,Hkv,d] uint8; Vt8 [B,Hkv,d,stride] uint8 as made by
    fp8_key_major. Returns O [B,Nq,Hq,d] bf16 and LSE [B,Hq,Nq] fp32."""
    import torch
    for t, nm in ((Q8, "Q8"), (K8, "K8"), (Vt8, "Vt8")):
        _need(t, nm, torch.uint8, None, Q8.device)
    if Q8.dim() != 4 or K8.dim() != 4 or Vt8.dim() != 4:
        raise ValueError("Q8 must be [B, Nq, Hq, d], K8 [B, Nk, Hkv, d], Vt8 [B, Hkv, d, stride]")
    B, Nq, Hq, d = Q8.shape
    Hkv = K8.shape[2]
    _need(K8, "K8", torch.uint8, (B, Nk, Hkv, d))
    if tuple(Vt8.shape[:3]) != (B, Hkv, d) or Vt8.shape[3] % 64 or Vt8.shape[3] < Nk:
        raise ValueError("Vt8 must be [B, Hkv, d, stride] with stride a multiple of 64 and at least Nk")
    O = _out(O, "O", (B, Nq, Hq, d), torch.bfloat16, Q8.device)
    LSE = _out(LSE, "LSE", (B, Hq, Nq), torch.float32, Q8.device)
    _check(fa_fp8_fwd_raw(_ptr(Q8), _ptr(K8), _ptr(Vt8), _ptr(O), _ptr(LSE), B, Hq, Hkv, Nq, Nk, d, Vt8.shape[3], scale,
                          descale_q, descale_k, descale_v, causal, _stream()))
    return O, LSE


def fa_varlen_cross_fwd(Q, K, V, cu_seqlens_q, cu_seqlens_k, max_seqlen_q: int, max_seqlen_k: int, scale: float,
                        causal: bool, O=None, LSE=None):
    """Packed ragged forward with two lengths. Q [Tq,Hq,d], K,V [Tk,Hkv,d] bf16; offsets int32 on the GPU."""
    import torch
    x = _packed(Q, K, V, cu_seqlens_q, cu_seqlens_k, allowed=(torch.bfloat16, torch.float16))
    O, LSE = _fwd_outputs(x, O, LSE)
    _check(fa_varlen_cross_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(cu_seqlens_q), _ptr(cu_seqlens_k),
                                   x.nseq, x.Tq, x.Tk, max_seqlen_q, max_seqlen_k, x.Hq, x.Hkv, x.d, scale, causal,
                                   _stream(), x.et == torch.float16))
    return O, LSE


def fa_varlen_cross_bwd(Q, K, V, O, dO, LSE, cu_seqlens_q, cu_seqlens_k, max_seqlen_q: int, max_seqlen_k: int,
                        scale: float, causal: bool, dQ=None, dK=None, dV=None, workspace=None):
    """Packed ragged backward with two lengths. Returns dQ [Tq,Hq,d], dK, dV [Tk,Hkv,d] bf16."""
    import torch
    x = _packed(Q, K, V, cu_seqlens_q, cu_seqlens_k, allowed=(torch.bfloat16, torch.float16))
    dQ, dK, dV = _bwd_tensors(x, O, dO, LSE, dQ, dK, dV)
    ws = _workspace(workspace, fa_varlen_bwd_workspace_bytes(x.Tq, x.Hq, x.Hkv, x.d), x.dev)
    _check(fa_varlen_cross_bwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK), _ptr(dV),
                                   _ptr(ws), _wsbytes(ws), _ptr(cu_seqlens_q), _ptr(cu_seqlens_k), x.nseq, x.Tq, x.Tk,
                                   max_seqlen_q, max_seqlen_k, x.Hq, x.Hkv, x.d, scale, causal, _stream(), x.et == torch.float16))
    return dQ, dK, dV


FA_SPLITKV_MAX_SPLITS = 128


def splitkv_default_splits(B, Hq, Hkv, Nq, Nk, ragged: bool = False) -> int:
    """About one workgroup per compute unit, and at least 8 blocks of 64 keys per share (measured:
    more, shorter shares cost more in prologues and in the merge than they gain in parallelism).
    ragged (a cache with a length of its own per sequence, Nk the capacity): the same for up to 128
    sequences in decoding shapes, where the decode kernel hands the sequences out longest first
    (measured on 64 sequences of 1 .. 8192 keys: 1 share 5.0 TB/s, 4 shares 4.3, 16 shares 2.5);
    otherwise about eight workgroups per compute unit and at least 16 blocks per share of a full
    cache, since more, shorter shares then even the load out (same batch in launch order: 4 shares
    3.7 TB/s, 1 share 2.6, 16 shares 2.9)."""
    units = B * Hkv * ((Nq * (Hq // Hkv) + 255) // 256)
    blocks = (Nk + 63) // 64
    if ragged and not (B <= 128 and Nq * (Hq // Hkv) <= 32):
        return max(1, min(FA_SPLITKV_MAX_SPLITS, blocks // 16, -(-2048 // units)))
    return max(1, min(FA_SPLITKV_MAX_SPLITS, blocks // 8, -(-256 // units)))


def fa_splitkv_fwd(Q, K, V, scale: float, causal: bool, num_splits: int = 0, O=None, LSE=None, workspace=None):
    """Few query rows against many keys; layouts and results as fa_cross_fwd. num_splits = 0 picks a default."""
    import torch
    x = _dense(Q, K, V)
    if num_splits <= 0:
        num_splits = splitkv_default_splits(x.B, x.Hq, x.Hkv, x.Nq, x.Nk)
    O, LSE = _fwd_outputs(x, O, LSE)
    ws = _workspace(workspace, fa_splitkv_fwd_workspace_bytes(x.B, x.Hq, x.Nq, x.d, num_splits), x.dev)
    _check(fa_splitkv_fwd_raw(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(ws), _wsbytes(ws), x.B, x.Hq, x.Hkv,
                              x.Nq, x.Nk, x.d, scale, causal, num_splits, _stream(), x.et == torch.float16))
    return O, LSE


def fa_kvcache_fwd(Q, Kcache, Vcache, scale: float, causal: bool, seqlens_k=None, block_table=None, max_seqlen_k: int = 0,
                   num_splits: int = 0, O=None, LSE=None, workspace=None):
    """Nq new queries per sequence, Q [B,Nq,Hq,d] bf16 or fp16, against a key/value cache of which sequence b
    uses its first seqlens_k[b] keys (int32 on the GPU; None: all). Contiguous cache: Kcache, Vcache
    [B,Nk,Hkv,d]. Paged: Kcache, Vcache [pages,page_size,Hkv,d] and block_table [B,pages_per_seq]
    int32 on the GPU; max_seqlen_k (0: pages_per_seq * page_size) bounds the lengths.
    Returns O [B,Nq,Hq,d] of that type and LSE [B,Hq,Nq] fp32. num_splits = 0 picks a default."""
    import torch
    et = _elem_type(Q)
    _need(Q, "Q", et)
    if Q.dim() != 4 or Kcache.dim() != 4:
        raise ValueError("Q must be [B, Nq, Hq, d] and the caches [B, Nk, Hkv, d] or [pages, page_size, Hkv, d]")
    x = _Dims()
    x.B, x.Nq, x.Hq, x.d = Q.shape
    x.Hkv, x.et, x.dev = Kcache.shape[2], et, Q.device
    _need(Kcache, "Kcache", x.et, None, x.dev)
    _need(Vcache, "Vcache", x.et, tuple(Kcache.shape), x.dev)
    if Kcache.shape[3] != x.d:
        raise ValueError("the caches must have the head dimension of Q")
    page_size = pages_per_seq = 0
    if block_table is None:
        if Kcache.shape[0] != x.B:
            raise ValueError("a contiguous cache must be [B, Nk, Hkv, d]")
        x.Nk = Kcache.shape[1]
    else:
        _need(block_table, "block_table", torch.int32, None, x.dev)
        if block_table.dim() != 2 or block_table.shape[0] != x.B:
            raise ValueError("block_table must be [B, pages_per_seq]")
        page_size, pages_per_seq = Kcache.shape[1], block_table.shape[1]
        x.Nk = max_seqlen_k if max_seqlen_k > 0 else page_size * pages_per_seq
    if seqlens_k is not None:
        _need(seqlens_k, "seqlens_k", torch.int32, (x.B,), x.dev)
    x.q_shape, x.l_shape = (x.B, x.Nq, x.Hq, x.d), (x.B, x.Hq, x.Nq)
    if num_splits <= 0:
        num_splits = splitkv_default_splits(x.B, x.Hq, x.Hkv, x.Nq, x.Nk, ragged=seqlens_k is not None)
    O, LSE = _fwd_outputs(x, O, LSE)
    ws = _workspace(workspace, fa_splitkv_fwd_workspace_bytes(x.B, x.Hq, x.Nq, x.d, num_splits), x.dev)
    _check(fa_kvcache_fwd_raw(_ptr(Q), _ptr(Kcache), _ptr(Vcache), _ptr(seqlens_k) if seqlens_k is not None else 0,
                              _ptr(block_table) if block_table is not None else 0, _ptr(O), _ptr(LSE), _ptr(ws),
                              _wsbytes(ws), x.B, x.Hq, x.Hkv, x.Nq, x.Nk, x.d, page_size, pages_per_seq, scale, causal,
                              num_splits, _stream(), et == torch.float16))
    return O, LSE


def fa_mfma_probe(iters: int, random_operands: bool):
    """Time the register-resident MFMA loop: returns (TFLOP/s, shader clock in GHz)."""
    import torch
    scratch = torch.zeros(fa_mfma_probe_scratch_bytes(), dtype=torch.uint8, device="cuda")
    _check(fa_mfma_probe_raw(max(1, iters // 10), random_operands, _ptr(scratch), _stream()))  # warm-up
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    _check(fa_mfma_probe_raw(iters, random_operands, _ptr(scratch), _stream()))
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    cycles, ticks = scratch[:16].view(torch.int64).tolist()
    flops = 256.0 * 8 * iters * 32 * 32768.0
    return flops / (ms * 1e-3) / 1e12, cycles / (ticks * 10.0)
