/*
 * fa.h - C ABI of the MI355X (gfx950) exact-attention library.
 *
 * The library computes scaled-dot-product attention
 *     O = softmax(scale * Q K^T [+ causal mask]) V
 * and its gradients tile by tile with an online softmax, so the N x N score and
 * probability matrices are never written to device memory (Algorithm 1 and
 * Algorithm 2 of the paper; problem statement in section 2.2).
 *
 * Conventions common to every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller. The library
 *     never allocates, frees or retains memory and never synchronises: work is
 *     enqueued on `stream` (a hipStream_t handle passed as void*, NULL = the
 *     default stream) and the call returns at once.
 *   - Element type of Q, K, V, O, dO, dQ, dK, dV is bfloat16 (2 bytes). LSE and
 *     the workspace are float32. All tensor pointers must be 16-byte aligned.
 *   - Dense layout (token-major, head dim contiguous, no padding):
 *         Q, O, dO, dQ : [B, N, Hq,  d]
 *         K, V, dK, dV : [B, N, Hkv, d]
 *         LSE          : [B, Hq, N]
 *     Packed ragged layout: the tokens of all sequences are concatenated,
 *     T = cu_seqlens[nseq]; sequence s owns rows cu_seqlens[s] .. cu_seqlens[s+1]-1:
 *         Q, O, dO, dQ : [T, Hq,  d]
 *         K, V, dK, dV : [T, Hkv, d]
 *         LSE          : [Hq, T]
 *   - Supported: d a multiple of 8, 8 <= d <= 128 (section 3.3 names 64-128 as the
 *     usual range), and d = 256. Up to 128 the kernels work on tiles 64 or 128 wide:
 *     other head dimensions are padded with zeros on chip (memory holds exactly d
 *     elements per row, nothing is read or written past them) and cost as much as the
 *     next tile width. d = 256 has kernels of its own. The dropout, mask and split-key
 *     entry points take d in {64, 128} only. Hq a positive
 *     multiple of Hkv (grouped-query
 *     attention: query head h reads key/value head h / (Hq/Hkv), paragraph
 *     "Multi-query attention and grouped-query attention" of section 3.1);
 *     scale > 0. fa_fwd, fa_bwd and fa_varlen_* take one length per sequence
 *     (self-attention); the fa_cross_*, fa_varlen_cross_* and fa_splitkv_* entry
 *     points take a query length and a key length.
 *   - causal != 0 masks score (r, c) with c > r inside each sequence
 *     (section 3.1.1, "Causal masking").
 *   - Return value: FA_OK or a negative FA_ERR_* code. Arguments are validated
 *     before anything is launched, so an error return means nothing ran.
 *     Inputs are never written. Outputs are fully overwritten (gradients are
 *     not accumulated into). Calls on different streams may overlap as long as
 *     they do not share output or workspace buffers.
 */
#ifndef FA_H_
#define FA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FA_OK 0
#define FA_ERR_NULL (-1)        /* a required pointer is NULL */
#define FA_ERR_SHAPE (-2)       /* non-positive dimension, Hq % Hkv != 0, scale <= 0 or not finite,
                                   inconsistent ragged description */
#define FA_ERR_UNSUPPORTED (-3) /* head dim neither a multiple of 8 in 8 .. 128 nor 256 (dropout, mask, split keys: not 64 or 128) */
#define FA_ERR_ALIGN (-4)       /* a tensor pointer is not 16-byte aligned */
#define FA_ERR_WORKSPACE (-5)   /* workspace smaller than fa_*_workspace_bytes() */
#define FA_ERR_LAUNCH (-6)      /* the HIP runtime refused a launch; see fa_last_hip_error() */

/* Library version: major * 10000 + minor * 100 + patch. */
int fa_version(void);

/* Static, NUL-terminated description of a status code. Never NULL. */
const char* fa_status_string(int status);

/* Numeric hipError_t of the most recent failed launch on this thread (0 if none). */
int fa_last_hip_error(void);

/*
 * Forward pass (Algorithm 1): O and the row-wise logsumexp
 *     LSE[b, h, r] = log sum_c exp(scale * q_r . k_c)   (natural log, masked columns excluded)
 * which is the only softmax statistic the backward pass needs (section 3.1.1,
 * second tweak). Dense layout.
 */
int fa_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
           int B, int Hq, int Hkv, int N, int d, float scale, int causal, void* stream);

/*
 * Backward pass (Algorithm 2). Needs the O and LSE that fa_fwd produced for the
 * same Q, K, V, scale and causal flag. Writes dQ, dK, dV (bfloat16).
 * `workspace` is device scratch of at least fa_bwd_workspace_bytes() bytes,
 * 16-byte aligned; its contents are undefined on entry and on return. It holds
 * D = rowsum(dO o O) (Algorithm 2, line 4). Two kernels are enqueued: a row-block
 * kernel that computes D for its rows and produces dQ by recomputing the
 * probabilities (instead of accumulating dQ across workgroups with atomic adds),
 * then a column-block kernel that produces dK and dV (section 3.2, "Backward
 * pass"). Head dimension 256 runs the D pre-pass as a launch of its own first.
 * All three outputs are bit-reproducible.
 */
size_t fa_bwd_workspace_bytes(int B, int Hq, int Hkv, int N, int d);
int fa_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
           const float* LSE, void* dQ, void* dK, void* dV,
           void* workspace, size_t workspace_bytes,
           int B, int Hq, int Hkv, int N, int d, float scale, int causal, void* stream);

/*
 * Profiling aid: the backward as three launches (D pre-pass, dK/dV kernel, dQ kernel)
 * restricted to a subset of them, so that each can be timed on its own. `stages`
 * is a bit mask; all three bits give the results of fa_bwd (which itself folds the
 * pre-pass into the dQ kernel: one launch and one pass over dO fewer). Both later stages read the D
 * the prep stage writes, so results are correct only if it ran first on the
 * same arguments. Same validation and errors as fa_bwd; stages == 0 or bits
 * outside the mask return FA_ERR_SHAPE.
 */
#define FA_STAGE_PREP 1 /* D = rowsum(dO o O) (Algorithm 2, line 4) */
#define FA_STAGE_DKDV 2 /* column-block loop: dK, dV (Algorithm 2, lines 5-19 without line 15) */
#define FA_STAGE_DQ 4   /* row-block loop: dQ (Algorithm 2, line 15) */
int fa_bwd_stages(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                  const float* LSE, void* dQ, void* dK, void* dV,
                  void* workspace, size_t workspace_bytes,
                  int B, int Hq, int Hkv, int N, int d, float scale, int causal, int stages,
                  void* stream);

/*
 * fa_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments, results
 * (bit for bit) and errors as fa_bwd, without `workspace`: D = rowsum(dO o O) goes to a
 * file-scope device array of FA_NOALLOC_MAX_ROWS floats (8 MiB) inside the library, which
 * every GPU the library has run on holds until the process ends. The call itself allocates
 * and frees nothing. B * N * Hq above FA_NOALLOC_MAX_ROWS returns FA_ERR_WORKSPACE and nothing
 * runs. The first call on a device looks the array's address up (hipGetSymbolAddress, with
 * that device current; a failure returns FA_ERR_LAUNCH, see fa_last_hip_error()): make that
 * first call outside graph capture. All calls on one GPU share the one array: calls that may
 * overlap on a GPU (different streams, or graphs replayed concurrently) race on it and must be
 * ordered by the caller; nothing in it needs clearing between calls (every call first
 * overwrites the part it then reads).
 */
#define FA_NOALLOC_MAX_ROWS (2 * 1024 * 1024)
int fa_bwd_noalloc(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                   const float* LSE, void* dQ, void* dK, void* dV,
                   int B, int Hq, int Hkv, int N, int d, float scale, int causal, void* stream);

/*
 * Packed ragged batch (not in the paper; each sequence is an independent
 * attention problem of Algorithm 1 / Algorithm 2). `cu_seqlens` is a DEVICE
 * array of nseq + 1 non-decreasing int32 offsets starting at 0;
 * `total_tokens` must equal cu_seqlens[nseq] and `max_seqlen` must be at least
 * the longest sequence (both are host-side copies the caller already has; the
 * library does not read the device array on the host). Empty sequences are
 * allowed. Rows of an output that belong to no sequence do not exist, so every
 * output row is written.
 */
int fa_varlen_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                  const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                  int Hq, int Hkv, int d, float scale, int causal, void* stream);

size_t fa_varlen_bwd_workspace_bytes(int total_tokens, int Hq, int Hkv, int d);
int fa_varlen_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                  const float* LSE, void* dQ, void* dK, void* dV,
                  void* workspace, size_t workspace_bytes,
                  const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                  int Hq, int Hkv, int d, float scale, int causal, void* stream);

/*
 * Two lengths: Nq query rows against Nk key/value rows per sequence (cross-attention, or the
 * newest Nq tokens against a key/value cache of Nk, the inference setting the multi-/grouped-
 * query paragraph of section 3.1.2 refers to). Section 2.2 defines S = QK^T for any two row
 * counts and Algorithms 1 and 2 never use that S is square; the causal mask of section 3.1.1
 * is only stated for Nq = Nk. Here query r stands at position r + Nk - Nq of the keys, i.e.
 * sees keys c <= r + Nk - Nq (Nq = Nk is the printed mask); causal with Nq > Nk would leave
 * rows without keys and returns FA_ERR_SHAPE.
 * Layout: Q, O, dO, dQ [B, Nq, Hq, d]; K, V, dK, dV [B, Nk, Hkv, d]; LSE [B, Hq, Nq];
 * everything else (ownership, alignment, errors, workspace, what is overwritten) as for
 * fa_fwd / fa_bwd, which are the case Nq = Nk = N. A few query rows against many keys run on
 * one workgroup per 256 query rows and head: the key sequence is not split across workgroups.
 */
int fa_cross_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                 int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal, void* stream);
size_t fa_cross_bwd_workspace_bytes(int B, int Hq, int Hkv, int Nq, int Nk, int d);
int fa_cross_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                 const float* LSE, void* dQ, void* dK, void* dV,
                 void* workspace, size_t workspace_bytes,
                 int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal, void* stream);

/*
 * The same two entry points for IEEE half precision (fp16) elements instead of bfloat16: every
 * 16-bit tensor (Q, K, V, O, dO, dQ, dK, dV) holds fp16; LSE and the workspace stay float32
 * (fa_cross_bwd_workspace_bytes). The paper's hardware argument (section 2.1) is made for
 * FP16/BF16 matrix units alike; the kernels differ only in the MFMA instruction and in how
 * float32 results are rounded. Nq = Nk gives plain self-attention. fp16 has a narrower
 * exponent range than bfloat16: scores and gradients beyond 65504 overflow, as in any fp16
 * implementation.
 */
int fa_cross_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                     int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal, void* stream);
int fa_cross_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                     const float* LSE, void* dQ, void* dK, void* dV,
                     void* workspace, size_t workspace_bytes,
                     int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal, void* stream);

/*
 * Dropout on P (named, without an algorithm, in the footnote of section 2.2): the same two
 * passes as fa_cross_fwd / fa_cross_bwd (bfloat16, dense layout, two lengths) with
 *     P_drop = keep o P / (1 - p)
 * in place of P in O = P V and in every derivative; LSE is that of the undropped scores and
 * D = rowsum(dO o O) as in Algorithm 2. `keep` is a pure function of (seed, sequence, head,
 * query, key), so the backward pass regenerates the mask of the forward pass from the same
 * `seed` and `p_drop`; nothing is stored. Generator (this library's definition): with
 * bh = sequence * Hq + head and 32-bit wrap-around arithmetic,
 *     x = (key / 4) * 0x9E3779B1 + query * 0x85EBCA77
 *         + ((seed mod 2^32) xor (seed >> 32) * 0x27D4EB2F xor bh * 0xC2B2AE3D)
 *     x ^= x >> 16;  x *= 0x7FEB352D;  x ^= x >> 15;  x *= 0x846CA68B;  x ^= x >> 16
 *     keep = byte (key mod 4) of x  >=  round(256 * p_drop)       (threshold capped at 255)
 * so the effective drop probability is a multiple of 1/256, and 1 / (1 - p) uses that
 * multiple. 0 <= p_drop < 1, otherwise FA_ERR_SHAPE; a threshold of 0 runs the plain kernels.
 * Workspace: fa_cross_bwd_workspace_bytes.
 */
int fa_dropout_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                   int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                   float p_drop, uint64_t seed, void* stream);
int fa_dropout_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                   const float* LSE, void* dQ, void* dK, void* dV,
                   void* workspace, size_t workspace_bytes,
                   int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                   float p_drop, uint64_t seed, void* stream);

/*
 * Dropout on P for packed ragged batches: fa_varlen_fwd / fa_varlen_bwd with the dropout of
 * fa_dropout_fwd / fa_dropout_bwd (same reading of the footnote of section 2.2, same generator;
 * the head index of the generator is bh = sequence * Hq + head, query and key are counted from
 * the start of their sequence, so a ragged batch of equal lengths drops exactly what the dense
 * batch drops). Layouts, arguments and workspace as for fa_varlen_fwd / fa_varlen_bwd
 * (fa_varlen_bwd_workspace_bytes); d in {64, 128}; bfloat16 elements.
 */
int fa_varlen_dropout_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                          const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                          int Hq, int Hkv, int d, float scale, int causal,
                          float p_drop, uint64_t seed, void* stream);
int fa_varlen_dropout_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                          const float* LSE, void* dQ, void* dK, void* dV,
                          void* workspace, size_t workspace_bytes,
                          const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                          int Hq, int Hkv, int d, float scale, int causal,
                          float p_drop, uint64_t seed, void* stream);

/*
 * Elementwise mask on S (section 2.2, the footnote to the definition of S, P, O, which names
 * masking without giving an algorithm). Reading taken here: a tensor M is ADDED to the scaled
 * scores, S = scale * Q K^T + M, before the causal rule (if any) and the softmax; the rest of
 * Algorithms 1 and 2 is unchanged, with P = exp(S - L) taken from these scores. Entries of M
 * are finite or -inf: -inf removes an entry (a boolean mask is M in {0, -inf}), finite values
 * act as a bias on the scores (relative-position biases and the like). +inf and NaN are not
 * allowed (not checked). A query row left without any entry gets O = 0 and L = -inf in the
 * forward pass and contributes nothing to dQ, dK, dV. M is an input of both passes and
 * receives no gradient.
 *
 * M (device, bfloat16, 16-byte aligned, never written) holds element (b, h, r, c) at
 *     M[b * mask_batch_stride + h * mask_head_stride + r * mask_row_stride + c]
 * (strides in elements). mask_batch_stride = 0 shares one mask over the sequences,
 * mask_head_stride = 0 over the query heads. All three strides are multiples of 8 and
 * mask_row_stride >= Nk rounded up to a multiple of 8 (rows are padded in memory; the pad is
 * read but never used), otherwise FA_ERR_SHAPE. Layouts, lengths and the causal rule as for
 * fa_cross_fwd / fa_cross_bwd; d in {64, 128}; bfloat16 elements; workspace as for
 * fa_cross_bwd (fa_cross_bwd_workspace_bytes).
 */
int fa_mask_fwd(const void* Q, const void* K, const void* V, const void* M, void* O, float* LSE,
                int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                long long mask_batch_stride, long long mask_head_stride, long long mask_row_stride,
                void* stream);
int fa_mask_bwd(const void* Q, const void* K, const void* V, const void* M, const void* O,
                const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                void* workspace, size_t workspace_bytes,
                int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                long long mask_batch_stride, long long mask_head_stride, long long mask_row_stride,
                void* stream);

/*
 * fa_mask_bwd that also returns the gradient of the mask, for a mask read as a learned bias (the
 * footnote of section 2.2 names masking and no more; with S = scale * Q K^T + M the derivative with
 * respect to M is Algorithm 2's dS = P o (dP - D), before the factor `scale` that dQ and dK carry).
 * dM (device, element type of Q, 16-byte aligned) receives entry (b, h, r, c) at
 *     dM[b * dmask_batch_stride + h * dmask_head_stride + r * dmask_row_stride + c]
 * for EVERY (sequence, query head), also when M itself is shared over sequences or heads (the
 * gradient of a shared mask is the sum of dM over what shares it, left to the caller). Strides in
 * elements, multiples of 8, dmask_row_stride >= Nk rounded up to 8, dmask_head_stride >= Nq rows,
 * dmask_batch_stride >= Hq heads (FA_ERR_SHAPE otherwise). Entries that M removes get 0. Up to three
 * elements of a row's padding past column Nk may be written (zeros). With causal = 1 the kernels
 * never visit blocks of 64 keys that lie wholly above a wavefront's 32 rows: those entries (all
 * zero) are NOT written, so pass dM zero-filled when the causal rule is on. Everything else,
 * dQ, dK, dV included, is fa_mask_bwd (or fa_mask_bwd_f16). Writing dM costs N_q x N_k elements of
 * HBM traffic per head, which the rest of the pass avoids.
 */
int fa_mask_bwd_dmask(const void* Q, const void* K, const void* V, const void* M, const void* O,
                      const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* dM,
                      void* workspace, size_t workspace_bytes,
                      int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                      long long mask_batch_stride, long long mask_head_stride, long long mask_row_stride,
                      long long dmask_batch_stride, long long dmask_head_stride,
                      long long dmask_row_stride, void* stream);
int fa_mask_bwd_dmask_f16(const void* Q, const void* K, const void* V, const void* M, const void* O,
                          const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* dM,
                          void* workspace, size_t workspace_bytes,
                          int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                          long long mask_batch_stride, long long mask_head_stride,
                          long long mask_row_stride, long long dmask_batch_stride,
                          long long dmask_head_stride, long long dmask_row_stride, void* stream);

/*
 * Local (sliding-window) attention (section 5, "Discussion and Future Directions", names local
 * attention as a pattern the method combines with; the block skipping of section 3.1.1,
 * "Causal masking", is what makes it cheap). Reading: with query r standing at position
 * q = r + Nk - Nq among the keys (the alignment of the causal rule), key c is visible to it iff
 *     q - window_left <= c <= q + window_right ;
 * a negative bound means no bound on that side. window_right = 0 with window_left < 0 is the
 * causal rule; window_left = W - 1, window_right = 0 is a causal window over the W newest keys.
 * Everything else is fa_cross_fwd / fa_cross_bwd: same layouts, workspace
 * (fa_cross_bwd_workspace_bytes), grouped heads, errors. Only blocks inside the band are
 * visited, so time is proportional to the band's area. Needs Nq <= Nk (FA_ERR_SHAPE otherwise:
 * a query would stand before the first key); every row then sees at least its own position.
 * bfloat16, d in {64, 128} (FA_ERR_UNSUPPORTED otherwise) unless the bounds reduce to plain or
 * causal attention.
 */
int fa_local_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                 int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale,
                 int window_left, int window_right, void* stream);
int fa_local_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                 const float* LSE, void* dQ, void* dK, void* dV,
                 void* workspace, size_t workspace_bytes,
                 int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale,
                 int window_left, int window_right, void* stream);

/*
 * Local attention over a packed ragged batch: fa_varlen_fwd / fa_varlen_bwd with the window of
 * fa_local_fwd / fa_local_bwd applied inside every sequence, positions counted from the sequence's
 * first token (one length per sequence, so query r stands at position r). Layouts, cu_seqlens,
 * max_seqlen, workspace (fa_varlen_bwd_workspace_bytes) and errors as for fa_varlen_fwd /
 * fa_varlen_bwd; window arguments as for fa_local_fwd. bfloat16, d in {64, 128}
 * (FA_ERR_UNSUPPORTED otherwise) unless the bounds reduce to plain or causal attention.
 */
int fa_varlen_local_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                        const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                        int Hq, int Hkv, int d, float scale,
                        int window_left, int window_right, void* stream);
int fa_varlen_local_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                        const float* LSE, void* dQ, void* dK, void* dV,
                        void* workspace, size_t workspace_bytes,
                        const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                        int Hq, int Hkv, int d, float scale,
                        int window_left, int window_right, void* stream);

/*
 * Block-sparse attention (section 5 names it beside local attention). Reading: `block_mask` holds
 * one byte per block of `block` x `block` entries of S, row blocks counted from query 0 and key
 * blocks from key 0; an entry of S takes part in the softmax iff its block's byte is non-zero
 * (and, if `causal`, the causal rule with the alignment of fa_cross_fwd keeps it). A row left
 * without entries gets O = 0, LSE = -inf and contributes to no gradient. `block_mask` is a DEVICE
 * array of bytes [Bm, Hm, ceil(Nq/block), ceil(Nk/block)], rows dense, addressed through the two
 * strides in bytes (0 shares the pattern over sequences or heads); it is read, never written.
 * `block` is a power of two, at least 64 (FA_ERR_SHAPE otherwise). Wavefronts skip the blocks
 * that the pattern removes from their rows (or keys), and a workgroup whose 256 rows (keys) keep
 * at most half of the key blocks (row tiles) inside its causal range visits only those, so time
 * falls with the density.
 * Otherwise as fa_cross_fwd / fa_cross_bwd (layouts, workspace, grouped heads, errors).
 * bfloat16, d in {64, 128}; at most 262144 keys and ceil(Nq/32) * (Hq/Hkv) <= 4096
 * (FA_ERR_UNSUPPORTED beyond).
 */
int fa_blocksparse_fwd(const void* Q, const void* K, const void* V, const void* block_mask,
                       void* O, float* LSE, int B, int Hq, int Hkv, int Nq, int Nk, int d,
                       float scale, int causal, int block,
                       long long mask_batch_stride, long long mask_head_stride, void* stream);
int fa_blocksparse_bwd(const void* Q, const void* K, const void* V, const void* block_mask,
                       const void* O, const void* dO, const float* LSE,
                       void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                       int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                       int block, long long mask_batch_stride, long long mask_head_stride,
                       void* stream);

/*
 * The dropout, mask, window and block-sparse entry points for IEEE half precision (fp16) elements:
 * each is its bfloat16 namesake with every 16-bit tensor (Q, K, V, O, dO, dQ, dK, dV, and the
 * elementwise mask M of the mask pair) holding fp16, as fa_cross_fwd_f16 / fa_cross_bwd_f16 are
 * to fa_cross_fwd / fa_cross_bwd (section 2.1 argues for FP16 and BF16 matrix units alike).
 * LSE, the workspace, the block pattern's bytes, the dropout generator and every reading stated
 * above are unchanged; so are arguments, limits and errors. An fp16 mask entry is finite (at most
 * 65504 in magnitude) or -inf.
 */
int fa_dropout_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                       int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                       float p_drop, uint64_t seed, void* stream);
int fa_dropout_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                       const float* LSE, void* dQ, void* dK, void* dV,
                       void* workspace, size_t workspace_bytes,
                       int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                       float p_drop, uint64_t seed, void* stream);
int fa_mask_fwd_f16(const void* Q, const void* K, const void* V, const void* M, void* O, float* LSE,
                    int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                    long long mask_batch_stride, long long mask_head_stride,
                    long long mask_row_stride, void* stream);
int fa_mask_bwd_f16(const void* Q, const void* K, const void* V, const void* M, const void* O,
                    const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                    void* workspace, size_t workspace_bytes,
                    int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                    long long mask_batch_stride, long long mask_head_stride,
                    long long mask_row_stride, void* stream);
int fa_local_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                     int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale,
                     int window_left, int window_right, void* stream);
int fa_local_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                     const float* LSE, void* dQ, void* dK, void* dV,
                     void* workspace, size_t workspace_bytes,
                     int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale,
                     int window_left, int window_right, void* stream);
int fa_blocksparse_fwd_f16(const void* Q, const void* K, const void* V, const void* block_mask,
                           void* O, float* LSE, int B, int Hq, int Hkv, int Nq, int Nk, int d,
                           float scale, int causal, int block,
                           long long mask_batch_stride, long long mask_head_stride, void* stream);
int fa_blocksparse_bwd_f16(const void* Q, const void* K, const void* V, const void* block_mask,
                           const void* O, const void* dO, const float* LSE,
                           void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                           int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                           int block, long long mask_batch_stride, long long mask_head_stride,
                           void* stream);

/*
 * Forward pass on FP8 operands (section 5, "Discussion and Future Directions", names FP8; the
 * convention is this library's). Q8 [B, Nq, Hq, d] and K8 [B, Nk, Hkv, d] hold OCP FP8 E4M3 bytes
 * (1 sign, 4 exponent, 3 significand bits, bias 7, largest finite value 448), token-major like the
 * 16-bit tensors. V is handed over KEY-MAJOR: Vt8 [B, Hkv, d, vt_stride] E4M3, element (b, g, t, c)
 * = V[b, c, g, t], `vt_stride` (bytes between rows) a multiple of 64 and at least Nk rounded up to
 * 64, the padding past Nk holding finite values (zeros). Each tensor has one float scale,
 * x = descale * x8, all three positive and finite (FA_ERR_SHAPE otherwise, as for a bad stride).
 * Computes O = softmax(scale * (descale_q Q8)(descale_k K8)^T [+ causal]) (descale_v V8) with
 * float32 accumulation and softmax statistics; the probabilities are rounded to E4M3 (times 2^8,
 * relative to the row's running maximum) as operands of the second product, the only error beyond
 * the bfloat16 rounding of O. O [B, Nq, Hq, d] is bfloat16, LSE [B, Hq, Nq] float32 (of the
 * dequantised, scaled scores). d in {64, 128}; grouped heads and two lengths as fa_cross_fwd
 * (causal needs Nq <= Nk). All pointers 16-byte aligned.
 */
int fa_fp8_fwd(const void* Q8, const void* K8, const void* Vt8, void* O, float* LSE,
               int B, int Hq, int Hkv, int Nq, int Nk, int d, long long vt_stride,
               float scale, float descale_q, float descale_k, float descale_v,
               int causal, void* stream);

/*
 * Two lengths in the packed ragged layout: sequence s owns query rows
 * cu_seqlens_q[s] .. cu_seqlens_q[s+1] of Q, O, dO, dQ [total_q, Hq, d] and key/value rows
 * cu_seqlens_k[s] .. cu_seqlens_k[s+1] of K, V, dK, dV [total_k, Hkv, d]; LSE is [Hq, total_q].
 * Both offset arrays are DEVICE arrays of nseq + 1 non-decreasing int32 starting at 0;
 * total_* and max_seqlen_* are the caller's host copies of their last entries and of (upper
 * bounds on) the longest sequences. Each sequence is an independent problem as for
 * fa_cross_fwd / fa_cross_bwd, with the same causal alignment. Under the causal mask every
 * sequence must have at least as many keys as queries: the library cannot see the device
 * arrays, so for a sequence that breaks this the outputs of that sequence are unspecified
 * (nothing outside the output tensors is touched). A sequence with queries but no keys at all
 * (either setting of `causal`) has no softmax: its rows get O = 0, LSE = -inf and dQ = 0, as rows
 * that an elementwise mask leaves without entries do, and nothing is read from K or V for it.
 * The backward workspace is that of fa_varlen_bwd for total_q tokens
 * (fa_varlen_bwd_workspace_bytes).
 */
int fa_varlen_cross_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                        const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int nseq,
                        int total_q, int total_k, int max_seqlen_q, int max_seqlen_k,
                        int Hq, int Hkv, int d, float scale, int causal, void* stream);
int fa_varlen_cross_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                        const float* LSE, void* dQ, void* dK, void* dV,
                        void* workspace, size_t workspace_bytes,
                        const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int nseq,
                        int total_q, int total_k, int max_seqlen_q, int max_seqlen_k,
                        int Hq, int Hkv, int d, float scale, int causal, void* stream);

/*
 * Forward pass for FEW query rows against MANY keys (decoding against a key/value cache):
 * same result and layout as fa_cross_fwd, but the key sequence of every (sequence, key/value
 * head) is cut into `num_splits` shares handled by different workgroups, and the Hq / Hkv
 * query heads that share a key/value head are packed into one row block, so K and V are read
 * once. Each share leaves a normalised partial O and its logsumexp (float32) in `workspace`;
 * a second launch combines them with the identity section 3.1.1 uses between blocks,
 * O = sum_k exp(L_k - L) O_k, L = log sum_k exp(L_k). Shares in which a row sees no key
 * contribute nothing. `workspace`: caller-owned DEVICE memory, 16-byte aligned, at least
 * fa_splitkv_fwd_workspace_bytes() bytes, undefined on entry and exit. 1 <= num_splits <=
 * FA_SPLITKV_MAX_SPLITS, otherwise FA_ERR_SHAPE; more shares than 64-key blocks leave the
 * extra ones empty. Results differ from fa_cross_fwd only by rounding (the partial sums are
 * combined in a different order). When the rows of one key/value head, Nq * (Hq / Hkv), number at
 * most 32 (decoding), a kernel of its own runs in which the wavefronts of a workgroup divide the
 * keys of the share among themselves instead of the rows; nothing changes for the caller.
 */
#define FA_SPLITKV_MAX_SPLITS 128
size_t fa_splitkv_fwd_workspace_bytes(int B, int Hq, int Nq, int d, int num_splits);
int fa_splitkv_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                   void* workspace, size_t workspace_bytes,
                   int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                   int num_splits, void* stream);

/*
 * Forward against a key/value cache (the inference setting that the multi-query / grouped-query
 * paragraph of section 3.1 refers to; a cache is storage: the arithmetic is fa_splitkv_fwd's).
 * Nq new queries per sequence, Q [B, Nq, Hq, d], attend to the first seqlens_k[b] keys of sequence
 * b's cache; under the causal rule query r stands at position r + seqlens_k[b] - Nq. seqlens_k is a
 * DEVICE array of B int32 (nullptr: every sequence holds Nk keys); values are clamped into 0 .. Nk.
 * A row that sees no key (an empty cache, or more queries than cached keys under the causal rule)
 * gets O = 0, LSE = -inf.
 *   block_table == nullptr: Kcache, Vcache [B, Nk, Hkv, d], one slab of Nk rows (the capacity)
 *     per sequence; page_size and pages_per_seq are ignored.
 *   block_table != nullptr: Kcache, Vcache [pages, page_size, Hkv, d] are pools of pages and
 *     block_table a DEVICE array [B, pages_per_seq] of int32 page numbers: key c of sequence b is
 *     row c mod page_size of page block_table[b][c / page_size]. page_size is a power of two, at
 *     least 64 (FA_ERR_UNSUPPORTED otherwise); pages_per_seq * page_size >= Nk, the largest length
 *     any sequence may have (FA_ERR_SHAPE otherwise). Entries past a sequence's last page are never
 *     read; the entries that are read must name pages inside the pools (not checked).
 * The key sequence of every (sequence, key/value head) is split over num_splits workgroups as in
 * fa_splitkv_fwd: same workspace (fa_splitkv_fwd_workspace_bytes), limits (d in {64, 128},
 * bfloat16, 1 <= num_splits <= FA_SPLITKV_MAX_SPLITS) and errors. Nothing is written to the caches.
 */
int fa_kvcache_fwd(const void* Q, const void* Kcache, const void* Vcache, const int32_t* seqlens_k,
                   const int32_t* block_table, void* O, float* LSE,
                   void* workspace, size_t workspace_bytes,
                   int B, int Hq, int Hkv, int Nq, int Nk, int d, int page_size, int pages_per_seq,
                   float scale, int causal, int num_splits, void* stream);

/*
 * The packed ragged entry points (one and two lengths, with dropout, with a window), the split-key
 * forward and the key/value cache forward for IEEE half precision (fp16) elements: each is its bfloat16 namesake with every
 * 16-bit tensor holding fp16, as fa_cross_fwd_f16 / fa_cross_bwd_f16 are to fa_cross_fwd /
 * fa_cross_bwd. LSE, workspaces, offset arrays, lengths, page tables, limits and errors are
 * unchanged.
 */
int fa_varlen_dropout_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                              const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                              int Hq, int Hkv, int d, float scale, int causal,
                              float p_drop, uint64_t seed, void* stream);
int fa_varlen_dropout_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                              const float* LSE, void* dQ, void* dK, void* dV,
                              void* workspace, size_t workspace_bytes,
                              const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                              int Hq, int Hkv, int d, float scale, int causal,
                              float p_drop, uint64_t seed, void* stream);
int fa_varlen_local_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                            const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                            int Hq, int Hkv, int d, float scale,
                            int window_left, int window_right, void* stream);
int fa_varlen_local_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                            const float* LSE, void* dQ, void* dK, void* dV,
                            void* workspace, size_t workspace_bytes,
                            const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                            int Hq, int Hkv, int d, float scale,
                            int window_left, int window_right, void* stream);
int fa_varlen_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                      const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                      int Hq, int Hkv, int d, float scale, int causal, void* stream);
int fa_varlen_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                      const float* LSE, void* dQ, void* dK, void* dV,
                      void* workspace, size_t workspace_bytes,
                      const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen,
                      int Hq, int Hkv, int d, float scale, int causal, void* stream);
int fa_varlen_cross_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                            const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int nseq,
                            int total_q, int total_k, int max_seqlen_q, int max_seqlen_k,
                            int Hq, int Hkv, int d, float scale, int causal, void* stream);
int fa_varlen_cross_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                            const float* LSE, void* dQ, void* dK, void* dV,
                            void* workspace, size_t workspace_bytes,
                            const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int nseq,
                            int total_q, int total_k, int max_seqlen_q, int max_seqlen_k,
                            int Hq, int Hkv, int d, float scale, int causal, void* stream);
int fa_splitkv_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                       void* workspace, size_t workspace_bytes,
                       int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                       int num_splits, void* stream);
int fa_kvcache_fwd_f16(const void* Q, const void* Kcache, const void* Vcache, const int32_t* seqlens_k,
                       const int32_t* block_table, void* O, float* LSE,
                       void* workspace, size_t workspace_bytes,
                       int B, int Hq, int Hkv, int Nq, int Nk, int d, int page_size, int pages_per_seq,
                       float scale, int causal, int num_splits, void* stream);

/*
 * Measurement aid, not part of either algorithm: a register-resident loop of the bf16 MFMA
 * the kernels are built on (v_mfma_f32_32x32x16_bf16), the "matmul throughput" the paper
 * sets the non-matmul work against (section 2.1, section 3.1), measured on this device
 * instead of read off a datasheet. 256 workgroups of 8 wavefronts each issue iters * 32
 * MFMAs (iters * 32 * 32768 FLOPs per wavefront); the caller times the launch.
 * `random_operands` = 0 uses constant operands, 1 pseudo-random bf16 bit patterns: under
 * the chip's power limit the sustained clock depends on it.
 * `scratch` is caller-owned DEVICE memory of at least fa_mfma_probe_scratch_bytes() bytes,
 * 16-byte aligned; on completion its first 16 bytes hold two int64: shader-clock cycles and
 * ticks of the constant 100 MHz counter spent in the loop by one wavefront (their ratio is
 * the shader clock). Errors: FA_ERR_NULL, FA_ERR_ALIGN, FA_ERR_SHAPE (iters < 1), FA_ERR_LAUNCH.
 */
size_t fa_mfma_probe_scratch_bytes(void);
int fa_mfma_probe(int iters, int random_operands, void* scratch, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FA_H_ */
