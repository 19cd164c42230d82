// Internal interface between the C ABI (fa_api.hip) and the kernel files.
#pragma once
#include "fa_common.h"

namespace fa {

struct FwdArgs {
  Problem p;
  const __bf16* Q;
  const __bf16* K;
  const __bf16* V;
  __bf16* O;
  float* LSE;
  // key sequence split over workgroups (0: not split): partial O [nsplit, tokens, Hq, d] and
  // partial logsumexp [nsplit] x (layout of LSE), float32, in caller-provided workspace
  int nsplit;
  float* Opart;
  float* Lpart;
  // key/value cache (split kernel only): sequence s attends to its first seqlens_k[s] keys (nullptr: all
  // p.Nk; values are clamped into 0 .. p.Nk). With a block table (nullptr: one slab of p.Nk rows per
  // sequence) K and V are pools of pages of 2^page_log2 rows (a multiple of 64) and key c of sequence s
  // is row c mod 2^page_log2 of page block_table[s * table_stride + (c >> page_log2)].
  const int32_t* seqlens_k;
  const int32_t* block_table;
  int page_log2, table_stride;
};

struct BwdArgs {
  Problem p;
  const __bf16* Q;
  const __bf16* K;
  const __bf16* V;
  const __bf16* O;
  const __bf16* dO;
  const float* LSE;
  __bf16* dQ;
  __bf16* dK;
  __bf16* dV;
  float* Dvec;   // workspace: rowsum(dO o O), laid out like LSE
  // gradient of the elementwise mask (mask instantiation of the dQ kernel only; nullptr: not asked for):
  // dM = dS in the element type, entry (s, h, r, c) at dM[s * dm_bs + h * dm_hs + r * dm_rs + c]
  __bf16* dM;
  long dm_bs, dm_hs, dm_rs;
};

// FP8 (E4M3) forward: Q, K one byte per element in the token-major layout, V key-major
// [B, Hkv, d, vt_stride]; p.scale is the softmax scaling times the scales of Q and K
struct Fp8Args {
  Problem p;
  const void* Q;
  const void* K;
  const void* Vt;
  __bf16* O;
  float* LSE;
  long vt_stride;   // bytes between the rows of V^T: a multiple of 64, at least Nk rounded up to 64
  float descale_v;
};

hipError_t launch_fwd(const FwdArgs& a, int d, int causal, hipStream_t st);
// split forward for at most 32 (query row, head of the group) pairs per key/value head (fa_decode.hip):
// writes the shares' partial results like the split kernel; d in {64, 128}
hipError_t launch_fwd_decode(const FwdArgs& a, int d, int causal, hipStream_t st);
hipError_t launch_fwd_fp8(const Fp8Args& a, int d, int causal, hipStream_t st);
// stages: bit 0 D pre-pass, bit 1 dK/dV kernel, bit 2 dQ kernel
hipError_t launch_bwd(const BwdArgs& a, int d, int causal, int stages, hipStream_t st);
// ragged batches with two lengths: O (or dQ) = 0 and L = -inf for the query rows of sequences without keys
hipError_t launch_keyless_rows(const Problem& p, __bf16* out, float* lse, hipStream_t st);
// head dimension 256 (fa_d256.hip): plain problems only (no split, dropout, mask)
hipError_t launch_fwd256(const FwdArgs& a, int causal, hipStream_t st);
hipError_t launch_bwd256(const BwdArgs& a, int causal, int stages, hipStream_t st);
// register-resident MFMA loop: sink gets workgroups * 512 floats, clocks two counters
hipError_t launch_mfma_probe(float* sink, long long* clocks, int workgroups, int iters, int random_operands,
                             hipStream_t st);

}  // namespace fa
