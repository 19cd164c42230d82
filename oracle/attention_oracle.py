"""Float64 CPU oracle for exact scaled-dot-product attention, forward and backward.

TEST INFRASTRUCTURE ONLY. Nothing in the product path may import this file;
only tests/, the smoke check and the benchmark's cpu_baseline leg call it.
It shares no code with the HIP kernels and imports nothing but numpy.

The tiled method of the paper reaches exactly (up to rounding order) the result
of the standard definition (section 2.2, "Standard Attention Implementation";
section 3.1.1 states that Algorithm 1 returns softmax(QK^T)V with no
approximation), so this oracle is that definition written out, materialising
the full score matrix S and probability matrix P per (sequence, query head):

    S = scale * Q K^T          (section 2.2; the scaling is the footnote there)
    S[r, c] = -inf for c > r   (causal mask, section 3.1.1 "Causal masking")
    P = softmax_rows(S),  L = rowmax(S) + log(rowsum(exp(S - rowmax(S))))
                               (L: the logsumexp of section 3.1.1, tweak 2)
    O = P V

and, given dO (section 2.2, backward equations; Algorithm 2 for D and dS):

    dV = P^T dO,  dP = dO V^T,  D = rowsum(dO o O),  dS = P o (dP - D)
    dQ = scale * dS K,  dK = scale * dS^T Q

Readings taken where the text is silent or inconsistent:
  * the backward equations are printed without the softmax scaling; the chain
    rule through S = scale*QK^T puts `scale` on dQ and dK;
  * section 2.2 prints dK = Q dS^T, which does not type-check for N x d
    operands; Algorithm 2's dS^T Q is used;
  * Algorithm 2 declares D in R^d; it has one entry per query row (R^N);
  * grouped-query attention (section 3.1.2 paragraph on MQA/GQA): query head h
    reads key/value head h // (Hq / Hkv); dK, dV are summed over the query
    heads of a group;
  * packed ragged batches are not in the paper: each sequence, delimited by
    cumulative offsets, is an independent attention problem;
  * a sequence of a ragged batch with queries but no keys has no softmax. Reading, the same
    as for a row that the elementwise mask leaves without entries (below): P = 0 on those rows,
    hence O = 0, L = -inf, and they contribute to no gradient;
  * two lengths (Nq queries against Nk keys; cross-attention, or the newest Nq
    tokens against a key/value cache, the inference setting the MQA/GQA
    paragraph of section 3.1.2 has in mind): section 2.2 defines S = QK^T for
    any two row counts; the causal mask of section 3.1.1 is stated for square S
    only. Reading: the queries are the LAST Nq positions of the Nk keys, so
    query r sits at position r + Nk - Nq and S[r, c] = -inf for
    c > r + Nk - Nq. Nq = Nk gives the printed mask. Causal with Nq > Nk would
    leave rows without any key and is rejected.

  * dropout on P (the footnote of section 2.2 names it; no algorithm is given):
    P_drop = keep o P / (1 - p) replaces P in O = P V and in its derivatives,
    while the logsumexp stays that of the undropped scores. `keep` comes from
    a counter-based generator of this build's own definition (dropout_keep
    below): one 32-bit hash per (head, query, group of 4 keys), one byte per
    key, kept when the byte is >= round(256 p). The drop probability is
    therefore a multiple of 1/256.

  * elementwise mask on S (the same footnote; no algorithm is given): a tensor M
    is ADDED to the scaled scores, S = scale * Q K^T + M, before the causal mask
    and the softmax. Entries of M are finite or -inf; -inf removes an entry
    (a boolean mask is M in {0, -inf}). M is a constant of the computation: it
    receives no gradient, and dQ, dK, dV follow from the same equations with
    the P of the masked scores. A row whose entries are all -inf has no
    softmax; reading: P = 0 on that row, hence O = 0, L = -inf, and the row
    contributes nothing to any gradient. M is [Bm, Hm, Nq, Nk] with Bm in
    {1, B} and Hm in {1, Hq} (size 1 = shared).
    Read as a learned bias M has a gradient of its own: dM = dS = P o (dP - D), the dS of
    Algorithm 2 before the factor `scale` (removed entries: 0).

  * local (sliding-window) and block-sparse attention (section 5 names them as patterns the
    method combines with; no definition is given). Reading: both only REMOVE entries of S
    before the softmax, exactly as the causal rule of section 3.1.1 does, and everything else
    is the standard definition on what is left.
      - window (left, right): query r stands at position p = r + Nk - Nq among the keys (the
        alignment of the causal rule) and sees the keys c with p - left <= c <= p + right;
        a negative bound means "unbounded on that side". right = 0, left < 0 is the causal
        rule; left = W - 1, right = 0 is a causal sliding window over the W newest keys.
      - block-sparse: a boolean matrix over (row block, key block) pairs of `block` x `block`
        entries, rows counted from query 0 and keys from key 0; an entry of S is kept iff
        its block is set (and the causal rule, if asked for, keeps it).
    A row left without entries has P = 0, O = 0, L = -inf, as with the elementwise mask.
    In a packed ragged batch the window applies inside each sequence, positions counted from
    the sequence's first token (one length per sequence, so p = r).

  * a key/value cache (section 3.1's multi-query paragraph speaks of the inference setting the
    two lengths exist for; no layout is given). Reading: a cache is storage, not arithmetic:
    sequence b attends to the first seqlens_k[b] keys of its cache, wherever they lie (one
    contiguous slab per sequence, or fixed-size pages named by a table), with the two-length
    definition above; rows that then see no key have P = 0.

  * FP8 operands (section 5 names FP8 as a direction; no algorithm is given). Reading: Q, K, V
    arrive quantised to OCP FP8 E4M3 (1 sign, 4 exponent, 3 significand bits, bias 7, largest
    finite value 448, no infinities) with one float scale per tensor, x = descale * x8; the
    computation is the standard definition on those dequantised values. What an
    implementation does with P on chip (the HIP path rounds it to E4M3 as an operand of the
    second product) is its own error, bounded in the tests, and no part of the definition.

Layouts: dense Q,O,dO,dQ [B, Nq, Hq, d]; K,V,dK,dV [B, Nk, Hkv, d]; L [B, Hq, Nq]
(Nq = Nk = N for self-attention).
Packed: Q.. [T, Hq, d]; K.. [T, Hkv, d]; L [Hq, T].
All arithmetic is float64. Every function here is pinned by tests/test_oracle_pins.py.
"""
import numpy as np


def widen_bf16(bits):
    """bfloat16 bit patterns (uint16) -> float64, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def widen_f16(bits):
    """IEEE half precision bit patterns (uint16) -> float64, exactly."""
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def widen_e4m3(bits):
    """OCP FP8 E4M3 bit patterns (uint8) -> float64, exactly: S EEEE MMM, bias 7;
    E = 0: subnormal M/8 * 2^-6; E = 15, M = 7: NaN; every other pattern a finite number."""
    b = np.ascontiguousarray(bits, dtype=np.uint8).astype(np.int64)
    sign = np.where(b & 0x80, -1.0, 1.0)
    e, m = (b >> 3) & 0xF, b & 0x7
    val = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    return sign * np.where((e == 15) & (m == 7), np.nan, val)


def attention_forward_fp8(Q8, K8, V8, descale_q, descale_k, descale_v, scale, causal):
    """Dense forward on E4M3 inputs with per-tensor scales: the definition on the dequantised
    values. Q8 [B,Nq,Hq,d], K8, V8 [B,Nk,Hkv,d] uint8. Returns O [B,Nq,Hq,d], L [B,Hq,Nq]."""
    return attention_forward(descale_q * widen_e4m3(Q8), descale_k * widen_e4m3(K8), descale_v * widen_e4m3(V8),
                             scale, causal)


def scores(q, k, scale, causal):
    """S for one head: q [Nq, d], k [Nk, d] -> [Nq, Nk] (section 2.2). Causal:
    query r is at position r + Nk - Nq; entries with a column index above
    that position are -inf (section 3.1.1 for Nq = Nk)."""
    s = scale * (q @ k.T)
    if causal:
        nq, nk = s.shape
        if nq > nk:
            raise ValueError("causal attention needs at least as many keys as queries")
        r = np.arange(nq)[:, None] + (nk - nq)
        c = np.arange(nk)[None, :]
        s = np.where(c > r, -np.inf, s)
    return s


def softmax_rows(s):
    """Row-wise softmax and logsumexp of a score matrix (section 2.2 and the
    logsumexp L of section 3.1.1)."""
    m = np.max(s, axis=1, keepdims=True)
    e = np.exp(s - m)
    l = np.sum(e, axis=1, keepdims=True)
    return e / l, (m + np.log(l))[:, 0]


def head_forward(q, k, v, scale, causal):
    """One head: returns O [N, d], L [N], P [N, N]."""
    p, lse = softmax_rows(scores(q, k, scale, causal))
    return p @ v, lse, p


def head_backward(q, k, v, do, scale, causal):
    """One head: returns dQ, dK, dV (section 2.2 backward; Algorithm 2 for the
    form dS = P o (dP - D) with D = rowsum(dO o O))."""
    o, _, p = head_forward(q, k, v, scale, causal)
    dv = p.T @ do
    dp = do @ v.T
    big_d = np.sum(do * o, axis=1, keepdims=True)
    ds = p * (dp - big_d)
    dq = scale * (ds @ k)
    dk = scale * (ds.T @ q)
    return dq, dk, dv


def _group(Hq, Hkv):
    if Hkv <= 0 or Hq % Hkv != 0:
        raise ValueError("Hq must be a positive multiple of Hkv")
    return Hq // Hkv


def attention_forward(Q, K, V, scale, causal):
    """Dense batch forward. Q [B,Nq,Hq,d], K,V [B,Nk,Hkv,d] float64.
    Returns O [B,Nq,Hq,d], L [B,Hq,Nq]."""
    B, N, Hq, d = Q.shape
    G = _group(Hq, K.shape[2])
    O = np.empty((B, N, Hq, d), dtype=np.float64)
    L = np.empty((B, Hq, N), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            o, lse, _ = head_forward(Q[b, :, h, :], K[b, :, g, :], V[b, :, g, :], scale, causal)
            O[b, :, h, :] = o
            L[b, h, :] = lse
    return O, L


def attention_backward(Q, K, V, dO, scale, causal):
    """Dense batch backward. Returns dQ [B,Nq,Hq,d], dK, dV [B,Nk,Hkv,d]."""
    B, N, Hq, d = Q.shape
    Hkv = K.shape[2]
    G = _group(Hq, Hkv)
    dQ = np.zeros((B, N, Hq, d), dtype=np.float64)
    dK = np.zeros(K.shape, dtype=np.float64)
    dV = np.zeros(V.shape, dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            dq, dk, dv = head_backward(Q[b, :, h, :], K[b, :, g, :], V[b, :, g, :],
                                       dO[b, :, h, :], scale, causal)
            dQ[b, :, h, :] = dq
            dK[b, :, g, :] += dk
            dV[b, :, g, :] += dv
    return dQ, dK, dV


def varlen_forward(Q, K, V, cu_seqlens, scale, causal, cu_seqlens_k=None):
    """Packed ragged forward. Q [T,Hq,d], K,V [Tk,Hkv,d]; returns O [T,Hq,d], L [Hq,T].
    Sequence s owns query rows cu_seqlens[s]:cu_seqlens[s+1] and key/value rows
    cu_seqlens_k[s]:cu_seqlens_k[s+1] (the same rows when cu_seqlens_k is None)."""
    T, Hq, d = Q.shape
    cu_k = cu_seqlens if cu_seqlens_k is None else cu_seqlens_k
    O = np.zeros((T, Hq, d), dtype=np.float64)
    L = np.zeros((Hq, T), dtype=np.float64)
    for s in range(len(cu_seqlens) - 1):
        a, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        ak, ek = int(cu_k[s]), int(cu_k[s + 1])
        if e == a:
            continue
        if ek == ak:  # queries without any key: no softmax; P = 0, so O = 0 and L = -inf
            L[:, a:e] = -np.inf
            continue
        o, lse = attention_forward(Q[None, a:e], K[None, ak:ek], V[None, ak:ek], scale, causal)
        O[a:e] = o[0]
        L[:, a:e] = lse[0]
    return O, L


def varlen_backward(Q, K, V, dO, cu_seqlens, scale, causal, cu_seqlens_k=None):
    """Packed ragged backward. Returns dQ [T,Hq,d], dK, dV [Tk,Hkv,d]."""
    cu_k = cu_seqlens if cu_seqlens_k is None else cu_seqlens_k
    dQ = np.zeros(Q.shape, dtype=np.float64)
    dK = np.zeros(K.shape, dtype=np.float64)
    dV = np.zeros(V.shape, dtype=np.float64)
    for s in range(len(cu_seqlens) - 1):
        a, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        ak, ek = int(cu_k[s]), int(cu_k[s + 1])
        if e == a or ek == ak:  # no queries: nothing flows to the keys; no keys: P = 0, dQ = 0
            continue
        dq, dk, dv = attention_backward(Q[None, a:e], K[None, ak:ek], V[None, ak:ek],
                                        dO[None, a:e], scale, causal)
        dQ[a:e], dK[ak:ek], dV[ak:ek] = dq[0], dk[0], dv[0]
    return dQ, dK, dV


# ---------------------------------------------------------------------------
# Sampled evaluation for full-size workloads: the same definition, restricted
# to chosen (sequence, query head) units or to chosen query rows, so a parity
# test can check a large GPU result without materialising every N x N matrix.
# ---------------------------------------------------------------------------

def rows_forward(q_rows, row_idx, k, v, scale, causal, nq=None):
    """Forward for selected query rows of one head: q_rows [R,d] are the rows
    `row_idx` of Q (which has `nq` rows; default: as many as there are keys);
    k, v [Nk,d]. Returns O rows [R,d] and L [R]."""
    s = scale * (q_rows @ k.T)
    if causal:
        nk = k.shape[0]
        c = np.arange(nk)[None, :]
        pos = np.asarray(row_idx)[:, None] + (nk - (nk if nq is None else nq))
        s = np.where(c > pos, -np.inf, s)
    p, lse = softmax_rows(s)
    return p @ v, lse


def head_statistics_blockwise(q, k, v, do, scale, causal, block=2048):
    """L [Nq], O [Nq, d] and D = rowsum(dO o O) [Nq] of one head, evaluated `block` query rows at a
    time so that no Nq x Nk matrix is ever held: the same definition as head_forward, row by row."""
    nq = q.shape[0]
    L = np.empty(nq)
    O = np.empty((nq, v.shape[1]))
    for a in range(0, nq, block):
        rows = np.arange(a, min(nq, a + block))
        O[rows], L[rows] = rows_forward(q[rows], rows, k, v, scale, causal, nq=nq)
    return L, O, np.sum(do * O, axis=1)


def rows_backward_dq(q_rows, row_idx, k, v, do_rows, scale, causal, nq=None):
    """dQ for selected query rows of one head (they need nothing from the other rows):
    dS_r = P_r o (dO_r V^T - D_r), D_r = dO_r . O_r, dQ_r = scale dS_r K."""
    s = scale * (q_rows @ k.T)
    if causal:
        nk = k.shape[0]
        pos = np.asarray(row_idx)[:, None] + (nk - (nk if nq is None else nq))
        s = np.where(np.arange(nk)[None, :] > pos, -np.inf, s)
    p, _ = softmax_rows(s)
    o = p @ v
    ds = p * (do_rows @ v.T - np.sum(do_rows * o, axis=1, keepdims=True))
    return scale * (ds @ k)


def cols_backward_dkdv(q, k_cols, v_cols, col_idx, nk, do, L, big_d, scale, causal):
    """dK and dV for selected key columns `col_idx` (of `nk` keys) of one head, given the row
    statistics L and D = rowsum(dO o O) of ALL query rows (head_statistics_blockwise):
    P[:, c] = exp(scale q . k_c - L) (0 where masked), dV_c = P[:, c]^T dO,
    dS[:, c] = P[:, c] o (dO v_c - D), dK_c = scale dS[:, c]^T Q."""
    nq = q.shape[0]
    p = np.exp(scale * (q @ k_cols.T) - L[:, None])  # [Nq, C]
    if causal:
        pos = np.arange(nq)[:, None] + (nk - nq)
        p = np.where(np.asarray(col_idx)[None, :] > pos, 0.0, p)
    ds = p * (do @ v_cols.T - big_d[:, None])
    return scale * (ds.T @ q), p.T @ do


# ---------------------------------------------------------------------------
# Dropout on P. The generator is defined here in plain integer arithmetic; the
# GPU kernels implement the same function on their own.
# ---------------------------------------------------------------------------

_M32 = 0xFFFFFFFF


def dropout_threshold(p_drop):
    """The 8-bit threshold for a drop probability: round(256 p), at most 255."""
    if not (0.0 <= p_drop < 1.0):
        raise ValueError("drop probability must be in [0, 1)")
    return min(255, int(round(256.0 * p_drop)))


def dropout_keep(seed, bh, nq, nk, threshold):
    """keep[r, c] for head index bh = b * Hq + h: boolean [nq, nk].

    key = (seed mod 2^32) xor (bh * 0xC2B2AE3D) xor (seed >> 32) * 0x27D4EB2F   (mod 2^32)
    x   = (c div 4) * 0x9E3779B1 + r * 0x85EBCA77 + key                        (mod 2^32)
    x  ^= x >> 16;  x *= 0x7FEB352D;  x ^= x >> 15;  x *= 0x846CA68B;  x ^= x >> 16
    keep = byte (c mod 4) of x  >=  threshold
    """
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    key = ((seed & _M32) ^ ((bh * 0xC2B2AE3D) & _M32) ^ (((seed >> 32) * 0x27D4EB2F) & _M32)) & _M32
    r = np.arange(nq, dtype=np.uint64)[:, None]
    c = np.arange(nk, dtype=np.uint64)[None, :]
    x = ((c >> np.uint64(2)) * np.uint64(0x9E3779B1) + r * np.uint64(0x85EBCA77) + np.uint64(key)) & np.uint64(_M32)
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x7FEB352D)) & np.uint64(_M32)
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x846CA68B)) & np.uint64(_M32)
    x ^= x >> np.uint64(16)
    byte = (x >> (np.uint64(8) * (c & np.uint64(3)))) & np.uint64(255)
    return byte >= np.uint64(threshold)


def head_forward_dropout(q, k, v, scale, causal, keep, threshold):
    """One head with dropout: O = (keep o P / (1 - t/256)) V; L as without dropout."""
    p, lse = softmax_rows(scores(q, k, scale, causal))
    rp = 256.0 / (256.0 - threshold)
    return (np.where(keep, p, 0.0) * rp) @ v, lse, p


def head_backward_dropout(q, k, v, do, scale, causal, keep, threshold):
    """One head with dropout: the chain rule through P_drop = keep o P * rp.
    dV = P_drop^T dO;  dP = keep o (dO V^T) * rp;  D = rowsum(dO o O) = rowsum(P o dP);
    dS = P o (dP - D);  dQ = scale dS K;  dK = scale dS^T Q."""
    o, _, p = head_forward_dropout(q, k, v, scale, causal, keep, threshold)
    rp = 256.0 / (256.0 - threshold)
    pd = np.where(keep, p, 0.0) * rp
    dv = pd.T @ do
    dp = np.where(keep, do @ v.T, 0.0) * rp
    big_d = np.sum(do * o, axis=1, keepdims=True)
    ds = p * (dp - big_d)
    return scale * (ds @ k), scale * (ds.T @ q), dv


def attention_forward_dropout(Q, K, V, scale, causal, p_drop, seed):
    """Dense batch forward with dropout. Shapes as attention_forward."""
    B, N, Hq, d = Q.shape
    G = _group(Hq, K.shape[2])
    t = dropout_threshold(p_drop)
    O = np.empty((B, N, Hq, d), dtype=np.float64)
    L = np.empty((B, Hq, N), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            keep = dropout_keep(seed, b * Hq + h, N, K.shape[1], t)
            o, lse, _ = head_forward_dropout(Q[b, :, h, :], K[b, :, h // G, :], V[b, :, h // G, :], scale, causal, keep, t)
            O[b, :, h, :] = o
            L[b, h, :] = lse
    return O, L


def attention_backward_dropout(Q, K, V, dO, scale, causal, p_drop, seed):
    """Dense batch backward with dropout. Shapes as attention_backward."""
    B, N, Hq, d = Q.shape
    G = _group(Hq, K.shape[2])
    t = dropout_threshold(p_drop)
    dQ = np.zeros(Q.shape, dtype=np.float64)
    dK = np.zeros(K.shape, dtype=np.float64)
    dV = np.zeros(V.shape, dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            keep = dropout_keep(seed, b * Hq + h, N, K.shape[1], t)
            dq, dk, dv = head_backward_dropout(Q[b, :, h, :], K[b, :, g, :], V[b, :, g, :], dO[b, :, h, :],
                                               scale, causal, keep, t)
            dQ[b, :, h, :] = dq
            dK[b, :, g, :] += dk
            dV[b, :, g, :] += dv
    return dQ, dK, dV


def varlen_forward_dropout(Q, K, V, cu_seqlens, scale, causal, p_drop, seed):
    """Packed ragged forward with dropout: every sequence is its own attention problem; the head
    index of the generator is sequence * Hq + head and rows and columns count from the start of
    the sequence, as in a dense batch. Q [T,Hq,d], K,V [T,Hkv,d]; returns O [T,Hq,d], L [Hq,T]."""
    T, Hq, d = Q.shape
    G = _group(Hq, K.shape[1])
    t = dropout_threshold(p_drop)
    O = np.zeros((T, Hq, d), dtype=np.float64)
    L = np.zeros((Hq, T), dtype=np.float64)
    for s in range(len(cu_seqlens) - 1):
        a, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        for h in range(Hq if e > a else 0):
            keep = dropout_keep(seed, s * Hq + h, e - a, e - a, t)
            o, lse, _ = head_forward_dropout(Q[a:e, h], K[a:e, h // G], V[a:e, h // G], scale, causal, keep, t)
            O[a:e, h] = o
            L[h, a:e] = lse
    return O, L


def varlen_backward_dropout(Q, K, V, dO, cu_seqlens, scale, causal, p_drop, seed):
    """Packed ragged backward with dropout. Returns dQ [T,Hq,d], dK, dV [T,Hkv,d]."""
    T, Hq, d = Q.shape
    G = _group(Hq, K.shape[1])
    t = dropout_threshold(p_drop)
    dQ = np.zeros(Q.shape, dtype=np.float64)
    dK = np.zeros(K.shape, dtype=np.float64)
    dV = np.zeros(V.shape, dtype=np.float64)
    for s in range(len(cu_seqlens) - 1):
        a, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        for h in range(Hq if e > a else 0):
            keep = dropout_keep(seed, s * Hq + h, e - a, e - a, t)
            dq, dk, dv = head_backward_dropout(Q[a:e, h], K[a:e, h // G], V[a:e, h // G], dO[a:e, h], scale, causal,
                                               keep, t)
            dQ[a:e, h] = dq
            dK[a:e, h // G] += dk
            dV[a:e, h // G] += dv
    return dQ, dK, dV


# ---------------------------------------------------------------------------
# Elementwise mask added to S (footnote of section 2.2; reading in the header)
# ---------------------------------------------------------------------------

def softmax_rows_masked(s):
    """softmax_rows for scores that may hold whole rows of -inf: such a row has
    P = 0 and L = -inf; every other row is the ordinary softmax."""
    m = np.max(s, axis=1, keepdims=True)
    dead = np.isneginf(m)
    e = np.exp(s - np.where(dead, 0.0, m))  # dead rows: exp(-inf) = 0 everywhere
    l = np.sum(e, axis=1, keepdims=True)
    p = e / np.where(dead, 1.0, l)
    lse = np.where(dead, -np.inf, m + np.log(np.where(dead, 1.0, l)))
    return p, lse[:, 0]


def head_forward_masked(q, k, v, mask, scale, causal):
    """One head with S = scale * Q K^T + mask (then the causal mask): O, L, P."""
    p, lse = softmax_rows_masked(scores(q, k, scale, causal) + mask)
    return p @ v, lse, p


def head_backward_masked(q, k, v, mask, do, scale, causal):
    """One head: dQ, dK, dV of section 2.2 / Algorithm 2 with the P of the masked scores."""
    o, _, p = head_forward_masked(q, k, v, mask, scale, causal)
    dv = p.T @ do
    dp = do @ v.T
    big_d = np.sum(do * o, axis=1, keepdims=True)
    ds = p * (dp - big_d)
    return scale * (ds @ k), scale * (ds.T @ q), dv


def head_backward_mask_gradient(q, k, v, mask, do, scale, causal):
    """One head: dM, the derivative of sum(O * dO) with respect to the mask added to the scaled
    scores. S = scale * Q K^T + M, so dM = dS = P o (dP - D) of Algorithm 2 (without the factor
    `scale` that dQ and dK carry). Entries that are removed (M = -inf, or above the causal
    diagonal) have P = 0 and so dM = 0: moving them by a finite amount changes nothing."""
    o, _, p = head_forward_masked(q, k, v, mask, scale, causal)
    dp = do @ v.T
    big_d = np.sum(do * o, axis=1, keepdims=True)
    return p * (dp - big_d)


def attention_backward_mask_gradient(Q, K, V, M, dO, scale, causal):
    """Dense batch: dM [B, Hq, Nq, Nk] for a mask with an entry of its own per (sequence, head)
    (M [B, Hq, Nq, Nk]; a shared mask's gradient would be the sum over what shares it)."""
    B, Nq, Hq, d = Q.shape
    G = _group(Hq, K.shape[2])
    if M.shape[0] != B or M.shape[1] != Hq:
        raise ValueError("the mask gradient is defined here for M [B, Hq, Nq, Nk]")
    dM = np.empty((B, Hq, Nq, K.shape[1]), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            dM[b, h] = head_backward_mask_gradient(Q[b, :, h], K[b, :, h // G], V[b, :, h // G], M[b, h], dO[b, :, h],
                                                   scale, causal)
    return dM


def _mask_of(M, b, h):
    return M[b if M.shape[0] > 1 else 0, h if M.shape[1] > 1 else 0]


def attention_forward_masked(Q, K, V, M, scale, causal):
    """Dense batch forward with an additive mask M [Bm, Hm, Nq, Nk] (Bm in {1, B}, Hm in {1, Hq})."""
    B, Nq, Hq, d = Q.shape
    G = _group(Hq, K.shape[2])
    O = np.empty((B, Nq, Hq, d), dtype=np.float64)
    L = np.empty((B, Hq, Nq), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            o, lse, _ = head_forward_masked(Q[b, :, h, :], K[b, :, g, :], V[b, :, g, :], _mask_of(M, b, h),
                                            scale, causal)
            O[b, :, h, :] = o
            L[b, h, :] = lse
    return O, L


def attention_backward_masked(Q, K, V, M, dO, scale, causal):
    """Dense batch backward with an additive mask: dQ, dK, dV (the mask receives no gradient)."""
    B, Nq, Hq, d = Q.shape
    G = _group(Hq, K.shape[2])
    dQ = np.zeros(Q.shape, dtype=np.float64)
    dK = np.zeros(K.shape, dtype=np.float64)
    dV = np.zeros(V.shape, dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            dq, dk, dv = head_backward_masked(Q[b, :, h, :], K[b, :, g, :], V[b, :, g, :], _mask_of(M, b, h),
                                              dO[b, :, h, :], scale, causal)
            dQ[b, :, h, :] = dq
            dK[b, :, g, :] += dk
            dV[b, :, g, :] += dv
    return dQ, dK, dV


# ---------------------------------------------------------------------------
# Local (sliding-window) and block-sparse patterns (section 5; reading in the header)
# ---------------------------------------------------------------------------

def window_visible(nq, nk, left, right):
    """[nq, nk] booleans: key c is visible to query r iff p - left <= c <= p + right with
    p = r + nk - nq; a negative bound is no bound."""
    p = np.arange(nq)[:, None] + (nk - nq)
    c = np.arange(nk)[None, :]
    vis = np.ones((nq, nk), dtype=bool)
    if left >= 0:
        vis &= c >= p - left
    if right >= 0:
        vis &= c <= p + right
    return vis


def block_visible(nq, nk, block_mask, block):
    """[nq, nk] booleans from a [ceil(nq/block), ceil(nk/block)] block mask."""
    bm = np.asarray(block_mask, dtype=bool)
    if bm.shape != (-(-nq // block), -(-nk // block)):
        raise ValueError("block mask must be [ceil(Nq/block), ceil(Nk/block)]")
    return np.repeat(np.repeat(bm, block, axis=0), block, axis=1)[:nq, :nk]


def head_forward_pattern(q, k, v, visible, scale, causal=False):
    """One head with the entries of S outside `visible` ([Nq, Nk] booleans) removed: O, L, P."""
    s = np.where(visible, scores(q, k, scale, causal), -np.inf)
    p, lse = softmax_rows_masked(s)
    return p @ v, lse, p


def head_backward_pattern(q, k, v, visible, do, scale, causal=False):
    """One head: dQ, dK, dV of section 2.2 / Algorithm 2 with the P of the remaining entries."""
    o, _, p = head_forward_pattern(q, k, v, visible, scale, causal)
    dv = p.T @ do
    dp = do @ v.T
    big_d = np.sum(do * o, axis=1, keepdims=True)
    ds = p * (dp - big_d)
    return scale * (ds @ k), scale * (ds.T @ q), dv


def _pattern_batch(Q, K, V, dO, scale, causal, visible_of):
    B, Nq, Hq, d = Q.shape
    G = _group(Hq, K.shape[2])
    O = np.empty((B, Nq, Hq, d), dtype=np.float64)
    L = np.empty((B, Hq, Nq), dtype=np.float64)
    dQ, dK, dV = np.zeros(Q.shape), np.zeros(K.shape), np.zeros(V.shape)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            vis = visible_of(b, h)
            o, lse, _ = head_forward_pattern(Q[b, :, h], K[b, :, g], V[b, :, g], vis, scale, causal)
            O[b, :, h], L[b, h] = o, lse
            if dO is not None:
                dq, dk, dv = head_backward_pattern(Q[b, :, h], K[b, :, g], V[b, :, g], vis, dO[b, :, h], scale, causal)
                dQ[b, :, h] = dq
                dK[b, :, g] += dk
                dV[b, :, g] += dv
    return O, L, dQ, dK, dV


def attention_forward_local(Q, K, V, scale, left, right):
    """Dense batch forward with the window (left, right): O [B,Nq,Hq,d], L [B,Hq,Nq]."""
    vis = window_visible(Q.shape[1], K.shape[1], left, right)
    return _pattern_batch(Q, K, V, None, scale, False, lambda b, h: vis)[:2]


def attention_backward_local(Q, K, V, dO, scale, left, right):
    """Dense batch backward with the window (left, right): dQ, dK, dV."""
    vis = window_visible(Q.shape[1], K.shape[1], left, right)
    return _pattern_batch(Q, K, V, dO, scale, False, lambda b, h: vis)[2:]


def varlen_forward_local(Q, K, V, cu_seqlens, scale, left, right):
    """Packed ragged forward with the window (left, right): every sequence is its own attention
    problem and positions count from its start. Q [T,Hq,d], K,V [T,Hkv,d]; returns O [T,Hq,d], L [Hq,T]."""
    T, Hq, d = Q.shape
    O = np.zeros((T, Hq, d), dtype=np.float64)
    L = np.zeros((Hq, T), dtype=np.float64)
    for s in range(len(cu_seqlens) - 1):
        a, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        if e > a:
            o, lse = attention_forward_local(Q[None, a:e], K[None, a:e], V[None, a:e], scale, left, right)
            O[a:e], L[:, a:e] = o[0], lse[0]
    return O, L


def varlen_backward_local(Q, K, V, dO, cu_seqlens, scale, left, right):
    """Packed ragged backward with the window (left, right): dQ [T,Hq,d], dK, dV [T,Hkv,d]."""
    dQ, dK, dV = np.zeros(Q.shape), np.zeros(K.shape), np.zeros(V.shape)
    for s in range(len(cu_seqlens) - 1):
        a, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        if e > a:
            dq, dk, dv = attention_backward_local(Q[None, a:e], K[None, a:e], V[None, a:e], dO[None, a:e], scale, left, right)
            dQ[a:e], dK[a:e], dV[a:e] = dq[0], dk[0], dv[0]
    return dQ, dK, dV


def kvcache_forward(Q, Kcache, Vcache, scale, causal, seqlens_k=None, block_table=None):
    """Forward of Nq new queries per sequence against a key/value cache (the inference setting of
    the multi-query paragraph of section 3.1; two lengths as in the header). Sequence b attends to
    the first seqlens_k[b] keys of its cache (all of them when seqlens_k is None); under the causal
    rule query r stands at position r + seqlens_k[b] - Nq. A row that sees no key (an empty cache,
    or more queries than keys under the causal rule) has P = 0: O = 0, L = -inf.
    Contiguous cache: Kcache, Vcache [B, Nk_max, Hkv, d]. Paged cache: Kcache, Vcache
    [pages, page_size, Hkv, d] and block_table [B, pages per sequence] of page numbers; key c of
    sequence b is row c % page_size of page block_table[b, c // page_size].
    Q [B, Nq, Hq, d] -> O [B, Nq, Hq, d], L [B, Hq, Nq]."""
    B, Nq, Hq, d = Q.shape
    G = _group(Hq, Kcache.shape[2])
    O = np.zeros((B, Nq, Hq, d), dtype=np.float64)
    L = np.full((B, Hq, Nq), -np.inf, dtype=np.float64)
    for b in range(B):
        if block_table is None:
            nk = Kcache.shape[1] if seqlens_k is None else int(seqlens_k[b])
            k, v = Kcache[b, :nk], Vcache[b, :nk]
        else:
            page = Kcache.shape[1]
            nk = block_table.shape[1] * page if seqlens_k is None else int(seqlens_k[b])
            rows = [(int(block_table[b, c // page]), c % page) for c in range(nk)]
            k = np.array([Kcache[pg, r] for pg, r in rows]).reshape(nk, Kcache.shape[2], d)
            v = np.array([Vcache[pg, r] for pg, r in rows]).reshape(nk, Vcache.shape[2], d)
        if nk == 0:
            continue
        vis = window_visible(Nq, nk, -1, 0) if causal else np.ones((Nq, nk), dtype=bool)
        for h in range(Hq):
            O[b, :, h], L[b, h], _ = head_forward_pattern(Q[b, :, h], k[:, h // G], v[:, h // G], vis, scale)
    return O, L


def attention_forward_blocksparse(Q, K, V, scale, causal, block_mask, block):
    """Dense batch forward with a block mask [Bm, Hm, ceil(Nq/block), ceil(Nk/block)]
    (Bm in {1, B}, Hm in {1, Hq}): O, L."""
    nq, nk = Q.shape[1], K.shape[1]
    return _pattern_batch(Q, K, V, None, scale, causal,
                          lambda b, h: block_visible(nq, nk, _mask_of(block_mask, b, h), block))[:2]


def attention_backward_blocksparse(Q, K, V, dO, scale, causal, block_mask, block):
    """Dense batch backward with a block mask: dQ, dK, dV."""
    nq, nk = Q.shape[1], K.shape[1]
    return _pattern_batch(Q, K, V, dO, scale, causal,
                          lambda b, h: block_visible(nq, nk, _mask_of(block_mask, b, h), block))[2:]
