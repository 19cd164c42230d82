"""Seeded synthetic inputs for the attention hot path.

This module holds no attention arithmetic: it only draws standard-normal
numbers with numpy's counter-based generator, rounds them to bfloat16 (round to
nearest, ties to even) and hands out the 16-bit patterns. Both the GPU parity
tests and the float64 CPU checker consume the same bit patterns, so neither
side ever sees a value the other did not.

The benchmark in the paper's "Benchmarking Attention" section is itself
synthetic (random Q, K, V at hidden size 2048, head dim 64 or 128, 16k tokens
in total); the recipes below reproduce those shapes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

__all__ = [
    "f32_to_bf16_bits",
    "f32_to_f16_bits",
    "f32_to_e4m3_bits",
    "make_fp8",
    "bf16_bits_to_f32",
    "AttnProblem",
    "make_dense",
    "make_cross",
    "make_varlen",
    "shape_only",
    "block_pattern",
    "cache_layout",
    "CONFIGS",
    "make_config",
]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (RNE) and return the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounding = ((u >> 16) & 1) + 0x7FFF
    out = ((u + rounding) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to IEEE half precision (RNE) and return the uint16 bit patterns."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to OCP FP8 E4M3 (round to nearest, ties to even; magnitudes beyond 448 saturate
    to 448) and return the uint8 bit patterns. Pure bit arithmetic: the spacing of E4M3 numbers at
    |x| in [2^e, 2^(e+1)) is 2^(e-3), and 2^-9 below 2^-6 (subnormals)."""
    x = np.ascontiguousarray(x, dtype=np.float32).astype(np.float64)
    a = np.minimum(np.abs(x), 448.0)
    e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.maximum(e, -6.0)
    step = np.exp2(e - 3)
    q = np.rint(a / step) * step  # numpy rounds halves to even
    q = np.minimum(q, 448.0)
    # encode
    eq = np.floor(np.log2(np.where(q > 0, q, 1.0)))
    sub = q < 2.0 ** -6
    expo = np.where(sub, 0, eq + 7).astype(np.int64)
    mant = np.where(sub, np.rint(q / 2.0 ** -9), np.rint((q / np.exp2(eq) - 1.0) * 8.0)).astype(np.int64)
    out = ((expo << 3) | mant).astype(np.uint8)
    out[np.signbit(x)] |= 0x80
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


@dataclass
class AttnProblem:
    """One attention problem: bf16 bit patterns plus its shape parameters.

    Dense layout: Q, dO are [B, N, Hq, d]; K, V are [B, Nk, Hkv, d] (Nk = N unless the
    problem has two lengths, `Nk` > 0).
    Packed ragged layout (cu_seqlens is not None): Q, dO are [T, Hq, d];
    K, V are [T, Hkv, d]; sequence s owns token rows cu_seqlens[s]:cu_seqlens[s+1].
    """

    name: str
    Q: np.ndarray
    K: np.ndarray
    V: np.ndarray
    dO: np.ndarray
    Hq: int
    Hkv: int
    d: int
    scale: float
    causal: bool
    B: int = 0
    N: int = 0
    Nk: int = 0
    dtype: str = "bf16"  # element type the 16-bit patterns encode: "bf16" or "f16"
    cu_seqlens: Optional[np.ndarray] = None
    seed: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def varlen(self) -> bool:
        return self.cu_seqlens is not None

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1]) if self.varlen else self.B * self.N

    @property
    def seqlens(self) -> np.ndarray:
        if self.varlen:
            return np.diff(self.cu_seqlens)
        return np.full(self.B, self.N, dtype=np.int64)

    @property
    def keys(self) -> int:
        """Key/value rows per sequence of a dense problem."""
        return self.Nk or self.N

    def fwd_flops(self) -> float:
        """Metric FLOPs of the forward pass: 4*N^2*d per query head and
        sequence, halved under the causal mask (the paper's benchmark formula).
        Two lengths: 4*d per visible (query, key) pair, Nq*Nk of them without
        the mask and Nq*Nk - Nq^2/2 with it (the same count for Nq = Nk)."""
        if self.meta.get("window") and not self.varlen:
            # sliding window: 4*d per visible (query, key) pair, counted exactly
            left, right = self.meta["window"]
            nk = self.keys
            pos = np.arange(self.N, dtype=np.int64) + (nk - self.N)
            lo = np.maximum(0, pos - left) if left >= 0 else np.zeros_like(pos)
            hi = np.minimum(nk - 1, pos + right) if right >= 0 else np.full_like(pos, nk - 1)
            return 4.0 * self.B * self.Hq * self.d * float(np.sum(hi - lo + 1))
        if self.meta.get("block_pattern") and not self.varlen:
            # block-sparse: 4*d per (query, key) pair of the kept blocks that the causal rule keeps too
            bp = self.meta["block_pattern"]
            bm = block_pattern(bp["seed"], 1, self.Hq, self.N, self.keys, bp["block"], bp["density"], self.causal)
            blk, nk = bp["block"], self.keys
            rows = np.arange(self.N, dtype=np.int64)
            pairs = 0.0
            for cb in range(bm.shape[3]):
                c0, c1 = cb * blk, min(nk, (cb + 1) * blk) - 1
                hi = np.minimum(c1, rows + (nk - self.N)) if self.causal else np.full_like(rows, c1)
                per_row = np.maximum(0, hi - c0 + 1)                       # visible keys of this key block per row
                per_rb = np.add.reduceat(per_row, np.arange(0, self.N, blk))  # ... per row block
                pairs += float(np.sum(bm[0, :, :, cb] * per_rb[None, :]))
            return 4.0 * self.B * self.d * pairs
        if self.Nk and not self.varlen:
            pairs = float(self.N) * self.Nk - (0.5 * float(self.N) ** 2 if self.causal else 0.0)
            return 4.0 * self.B * self.Hq * self.d * pairs
        n2 = float(np.sum(self.seqlens.astype(np.float64) ** 2))
        f = 4.0 * self.Hq * self.d * n2
        return f / 2.0 if self.causal else f

    def bwd_flops(self) -> float:
        return 2.5 * self.fwd_flops()


def _draw(rng: np.random.Generator, shape, mult: float = 1.0, dtype: str = "bf16") -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if mult != 1.0:
        x = x * np.float32(mult)
    return f32_to_f16_bits(x) if dtype == "f16" else f32_to_bf16_bits(x)


def make_dense(B, N, Hq, Hkv, d, causal, seed, scale=None, qk_mult=1.0,
               name="dense") -> AttnProblem:
    """Draw Q, K, V, dO (in that order) i.i.d. N(0,1), optionally scaling Q and
    K by `qk_mult` before the bf16 rounding."""
    rng = np.random.default_rng(seed)
    Q = _draw(rng, (B, N, Hq, d), qk_mult)
    K = _draw(rng, (B, N, Hkv, d), qk_mult)
    V = _draw(rng, (B, N, Hkv, d))
    dO = _draw(rng, (B, N, Hq, d))
    return AttnProblem(name=name, Q=Q, K=K, V=V, dO=dO, Hq=Hq, Hkv=Hkv, d=d,
                       scale=float(scale if scale is not None else d ** -0.5),
                       causal=bool(causal), B=B, N=N, seed=seed,
                       meta={"qk_mult": float(qk_mult), "standard_normal": qk_mult <= 1.0})


def make_cross(B, Nq, Nk, Hq, Hkv, d, causal, seed, scale=None, name="cross", dtype="bf16") -> AttnProblem:
    """Two lengths: Nq query rows against Nk key/value rows; Q, K, V, dO drawn in that order,
    rounded to bfloat16 or (dtype="f16") to IEEE half precision."""
    rng = np.random.default_rng(seed)
    Q = _draw(rng, (B, Nq, Hq, d), dtype=dtype)
    K = _draw(rng, (B, Nk, Hkv, d), dtype=dtype)
    V = _draw(rng, (B, Nk, Hkv, d), dtype=dtype)
    dO = _draw(rng, (B, Nq, Hq, d), dtype=dtype)
    return AttnProblem(name=name, Q=Q, K=K, V=V, dO=dO, Hq=Hq, Hkv=Hkv, d=d,
                       scale=float(scale if scale is not None else d ** -0.5),
                       causal=bool(causal), B=B, N=Nq, Nk=Nk, seed=seed, dtype=dtype)


def make_fp8(B, Nq, Nk, Hq, Hkv, d, causal, seed, scale=None, name="fp8") -> AttnProblem:
    """FP8 forward problem: Q, K, V drawn i.i.d. N(0,1) (in that order), each divided by its scale
    descale = max|x| / 448 (the usual amax scaling) and rounded to E4M3. The patterns are in
    Q, K, V (uint8); meta holds the three scales."""
    rng = np.random.default_rng(seed)
    out, scales = [], []
    for shape in ((B, Nq, Hq, d), (B, Nk, Hkv, d), (B, Nk, Hkv, d)):
        x = rng.standard_normal(size=shape, dtype=np.float32)
        ds = float(np.max(np.abs(x))) / 448.0
        out.append(f32_to_e4m3_bits(x / np.float32(ds)))
        scales.append(ds)
    return AttnProblem(name=name, Q=out[0], K=out[1], V=out[2], dO=None, Hq=Hq, Hkv=Hkv, d=d,
                       scale=float(scale if scale is not None else d ** -0.5), causal=bool(causal), B=B, N=Nq,
                       Nk=Nk if Nk != Nq else 0, seed=seed, dtype="e4m3", meta={"descale": tuple(scales)})


def make_varlen(seqlens, Hq, Hkv, d, causal, seed, scale=None,
                name="varlen", dtype="bf16") -> AttnProblem:
    """Packed ragged batch: tokens of all sequences concatenated."""
    seqlens = np.asarray(seqlens, dtype=np.int64)
    cu = np.zeros(len(seqlens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seqlens)
    T = int(cu[-1])
    rng = np.random.default_rng(seed)
    Q = _draw(rng, (T, Hq, d), dtype=dtype)
    K = _draw(rng, (T, Hkv, d), dtype=dtype)
    V = _draw(rng, (T, Hkv, d), dtype=dtype)
    dO = _draw(rng, (T, Hq, d), dtype=dtype)
    return AttnProblem(name=name, Q=Q, K=K, V=V, dO=dO, Hq=Hq, Hkv=Hkv, d=d,
                       scale=float(scale if scale is not None else d ** -0.5),
                       causal=bool(causal), cu_seqlens=cu, seed=seed, dtype=dtype,
                       meta={"max_seqlen": int(seqlens.max()) if len(seqlens) else 0})


# Named workloads. Seeds are 1000 + index of the workload family.
CONFIGS = {
    "tiny": dict(kind="dense", B=1, N=128, Hq=2, Hkv=2, d=64, causal=False, seed=1001),
    "d128_n8k_causal": dict(kind="dense", B=2, N=8192, Hq=16, Hkv=16, d=128, causal=True, seed=1003),
    "long_n16k_causal_x3": dict(kind="dense", B=1, N=16384, Hq=16, Hkv=16, d=128, causal=True,
                                seed=1004, qk_mult=3.0),
    "gqa_ragged": dict(kind="varlen", nseq=16, lo=256, hi=4096, Hq=32, Hkv=8, d=128, causal=True,
                       seed=1005),
    # two lengths: a chunk of 512 new tokens against a cache of 8192 keys, and plain cross-attention
    "chunk_512_on_8k": dict(kind="cross", B=8, Nq=512, Nk=8192, Hq=32, Hkv=8, d=128, causal=True, seed=1006),
    "cross_2k_on_8k": dict(kind="cross", B=4, Nq=2048, Nk=8192, Hq=16, Hkv=16, d=128, causal=False, seed=1007),
    # decoding: one new token per sequence against a cache of 8192 keys, grouped heads (forward only)
    "decode_b8_on_8k": dict(kind="cross", B=8, Nq=1, Nk=8192, Hq=32, Hkv=8, d=128, causal=True, seed=1008),
    "decode_b1_on_128k": dict(kind="cross", B=1, Nq=1, Nk=131072, Hq=32, Hkv=8, d=128, causal=True, seed=1009),
    # a serving batch: 64 sequences with 1 .. 8192 cached keys each, the caches cut into pages of 256 keys
    "decode_paged_b64_to_8k": dict(kind="cross", B=64, Nq=1, Nk=8192, Hq=32, Hkv=8, d=128, causal=True, seed=1030,
                                   cache=dict(page=256, seed=18600)),
    # half precision elements, the shape of d128_n8k_causal
    "f16_d128_n8k_causal": dict(kind="cross", B=2, Nq=8192, Nk=8192, Hq=16, Hkv=16, d=128, causal=True, seed=1010,
                                dtype="f16"),
    # head dimensions that the kernels pad on chip, 16k tokens and about 2048 hidden units
    "d96_n8k_causal": dict(kind="dense", B=2, N=8192, Hq=20, Hkv=20, d=96, causal=True, seed=1011),
    "d32_n8k_causal": dict(kind="dense", B=2, N=8192, Hq=64, Hkv=64, d=32, causal=True, seed=1012),
    "d256_n8k_causal": dict(kind="dense", B=2, N=8192, Hq=8, Hkv=8, d=256, causal=True, seed=1014),
    "d256_n8k_full": dict(kind="dense", B=2, N=8192, Hq=8, Hkv=8, d=256, causal=False, seed=1015),
    "d256_n2k_causal": dict(kind="dense", B=8, N=2048, Hq=8, Hkv=8, d=256, causal=True, seed=1016),
    # dropout on P (p = 0.1) and an elementwise mask (a bias on 70 % of the entries, 30 % removed,
    # one mask per sequence and head, drawn on the GPU from the given seed) on the benchmark shape
    "dropout_d128_n8k_causal": dict(kind="dense", B=2, N=8192, Hq=16, Hkv=16, d=128, causal=True, seed=1017,
                                    dropout=(0.1, 0x5EED0D12)),
    "dropout_d128_n8k_full": dict(kind="dense", B=2, N=8192, Hq=16, Hkv=16, d=128, causal=False, seed=1018,
                                  dropout=(0.1, 0x5EED0D12)),
    "dropout_gqa_ragged": dict(kind="varlen", nseq=16, lo=256, hi=4096, Hq=32, Hkv=8, d=128, causal=True, seed=1005,
                               dropout=(0.1, 0x5EED0D12)),
    "mask_d128_n8k_causal": dict(kind="dense", B=2, N=8192, Hq=16, Hkv=16, d=128, causal=True, seed=1019,
                                 mask=dict(seed=9800, removed=0.3)),
    "mask_d128_n8k_full": dict(kind="dense", B=2, N=8192, Hq=16, Hkv=16, d=128, causal=False, seed=1020,
                               mask=dict(seed=9801, removed=0.3)),
    # local attention: a causal window over the newest 1024 (2048) keys, and a two-sided window
    "local_d128_n8k_w1024": dict(kind="dense", B=2, N=8192, Hq=16, Hkv=16, d=128, causal=False, seed=1022, window=(1023, 0)),
    "local_d128_n16k_w2048": dict(kind="dense", B=1, N=16384, Hq=16, Hkv=16, d=128, causal=False, seed=1023, window=(2047, 0)),
    "local_d64_n8k_w512x2": dict(kind="dense", B=2, N=8192, Hq=32, Hkv=32, d=64, causal=False, seed=1024, window=(512, 512)),
    # FP8 (E4M3) operands, forward only: the benchmark shape and the long non-causal one
    "fp8_d128_n8k_causal": dict(kind="fp8", B=2, Nq=8192, Nk=8192, Hq=16, Hkv=16, d=128, causal=True, seed=1027),
    "fp8_d128_n16k_full": dict(kind="fp8", B=1, Nq=16384, Nk=16384, Hq=16, Hkv=16, d=128, causal=False, seed=1028),
    "fp8_d64_n8k_causal": dict(kind="fp8", B=2, Nq=8192, Nk=8192, Hq=32, Hkv=32, d=64, causal=True, seed=1029),
    # block-sparse: blocks of 128 x 128, half of them kept (one pattern per head), under the causal rule
    "blocksparse_d128_n8k_causal_half": dict(kind="dense", B=2, N=8192, Hq=16, Hkv=16, d=128, causal=True, seed=1025,
                                             block_pattern=dict(seed=17600, block=128, density=0.5)),
    "blocksparse_d128_n8k_causal_eighth": dict(kind="dense", B=2, N=8192, Hq=16, Hkv=16, d=128, causal=True, seed=1026,
                                               block_pattern=dict(seed=17601, block=128, density=0.125)),
    "mask_d64_n8k_full": dict(kind="dense", B=2, N=8192, Hq=32, Hkv=32, d=64, causal=False, seed=1021,
                              mask=dict(seed=9802, removed=0.3)),
}


def sweep_name(d: int, N: int, causal: bool) -> str:
    return f"sweep_d{d}_n{N}_{'causal' if causal else 'full'}"


for _d, _H in ((64, 32), (128, 16)):
    for _N in (512, 1024, 2048, 4096, 8192, 16384):
        for _c in (False, True):
            CONFIGS[sweep_name(_d, _N, _c)] = dict(kind="dense", B=16384 // _N, N=_N, Hq=_H, Hkv=_H,
                                                   d=_d, causal=_c, seed=1002)


def block_pattern(seed: int, Bm: int, Hm: int, nq: int, nk: int, block: int, density: float, causal: bool) -> np.ndarray:
    """A seeded block-sparse pattern [Bm, Hm, ceil(nq/block), ceil(nk/block)] of booleans: every block
    kept with probability `density`; the first key block and (causal) the diagonal block of every row
    block always, so that no row is left without keys."""
    g = np.random.default_rng(seed)
    bm = g.random((Bm, Hm, -(-nq // block), -(-nk // block))) < density
    bm[..., 0] = True
    if causal:
        for rb in range(bm.shape[2]):
            bm[:, :, rb, min((rb * block + nk - nq) // block, bm.shape[3] - 1)] = True
    return bm


def cache_layout(seed: int, B: int, capacity: int, page: int):
    """Per-sequence key counts, uniform in 1 .. capacity (the first sequence full, the second holding
    one key), and a page table [B, capacity / page] over a shuffled pool: (lengths, table)."""
    g = np.random.default_rng(seed)
    lens = g.integers(1, capacity + 1, B)
    lens[0] = capacity
    if B > 1:
        lens[1] = 1
    pps = -(-capacity // page)
    return lens.astype(np.int32), g.permutation(B * pps).reshape(B, pps).astype(np.int32)


def ragged_lengths(seed: int, nseq: int, lo: int, hi: int) -> np.ndarray:
    """Sequence lengths uniform in [lo, hi], drawn before the tensors from a
    generator of their own so they do not depend on the tensor shapes."""
    return np.random.default_rng(seed + 7919).integers(lo, hi + 1, nseq)


def shape_only(B, N, Hq, Hkv, d, causal, name, scale=None) -> AttnProblem:
    """A dense problem without host tensors, for callers that draw their inputs on the GPU and only
    need the shape and the FLOP count."""
    return AttnProblem(name=name, Q=None, K=None, V=None, dO=None, Hq=Hq, Hkv=Hkv, d=d,
                       scale=float(scale if scale is not None else d ** -0.5), causal=bool(causal), B=B, N=N)


def make_config(name: str) -> AttnProblem:
    c = dict(CONFIGS[name])
    kind = c.pop("kind")
    options = {k: c.pop(k) for k in ("dropout", "mask", "window", "block_pattern", "cache") if k in c}  # entry-point options, not part of the draw
    if kind == "dense":
        prob = make_dense(name=name, **c)
    elif kind == "cross":
        prob = make_cross(name=name, **c)
    elif kind == "fp8":
        prob = make_fp8(name=name, **c)
    else:
        lens = ragged_lengths(c["seed"], c.pop("nseq"), c.pop("lo"), c.pop("hi"))
        prob = make_varlen(lens, name=name, **c)
    prob.meta.update(options)
    return prob
