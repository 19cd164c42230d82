// C ABI of the attention library: argument validation, workspace carving, launches.
#include "../../include/fa.h"
#include "fa_kernels.h"

#include <atomic>
#include <cmath>
#include <cstdlib>

// Scratch of fa_bwd_noalloc: D = rowsum(dO o O) for up to FA_NOALLOC_MAX_ROWS (query row, head)
// pairs. Every GPU the library runs on holds its own copy of this array, at its own address,
// until the process ends. In host code the name below is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) float scratch[FA_NOALLOC_MAX_ROWS];

namespace {

// device address of `scratch` on each GPU, looked up once per device
constexpr int kMaxDevices = 64;
std::atomic<float*> g_scratch[kMaxDevices];

// 0 and the address, or a negative status (and the HIP error kept for fa_last_hip_error)
int scratch_on_current_device(float** out, int* hip_error) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
  if (e == hipSuccess) {
    float* p = g_scratch[dev].load(std::memory_order_acquire);
    if (!p) {  // first call on this device (two threads racing here look up the same address)
      void* sym = nullptr;
      e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
      if (e == hipSuccess && !sym) e = hipErrorInvalidSymbol;
      if (e == hipSuccess) {
        p = (float*)sym;
        g_scratch[dev].store(p, std::memory_order_release);
      }
    }
    if (e == hipSuccess) {
      *out = p;
      return FA_OK;
    }
  }
  *hip_error = (int)e;
  return FA_ERR_LAUNCH;
}

thread_local int g_last_hip_error = 0;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// any_d: the entry point also takes head dimensions that the kernels pad on chip
// (multiples of 8 up to 128) and 256, which has kernels of its own; otherwise only the two
// tile widths 64 and 128 themselves.
int check_common(int Hq, int Hkv, int d, float scale, bool any_d = true) {
  if (Hq <= 0 || Hkv <= 0 || d <= 0) return FA_ERR_SHAPE;
  if (Hq % Hkv != 0) return FA_ERR_SHAPE;
  if (!(scale > 0.f) || !std::isfinite(scale)) return FA_ERR_SHAPE;
  if (any_d ? ((d % 8 != 0 || d > 128) && d != 256) : (d != 64 && d != 128)) return FA_ERR_UNSUPPORTED;
  return FA_OK;
}

fa::Problem make_problem(const int32_t* cu, int nseq, int N, int Nk, int Hq, int Hkv, int d, long total, float scale,
                         const int32_t* cu_k = nullptr, int f16 = 0) {
  fa::Problem p;
  p.d = d;
  p.f16 = f16;
  p.drop_thr = 0;
  p.drop_seed = 0;
  p.drop_rp = 1.f;
  p.mask = nullptr;
  p.mask_bs = p.mask_hs = p.mask_rs = 0;
  p.win_left = p.win_right = -1;
  p.bmask = nullptr;
  p.bmask_bs = p.bmask_hs = 0;
  p.bmask_cols = p.bmask_log2 = 0;
  p.cu_seqlens = cu;
  p.cu_seqlens_k = cu_k;
  p.nseq = nseq;
  p.N = N;
  p.Nk = Nk;
  p.Hq = Hq;
  p.Hkv = Hkv;
  p.G = Hq / Hkv;
  p.total_tokens = (int)total;
  p.lse_seq_stride = cu ? 0 : (long)Hq * N;
  p.lse_head_stride = cu ? total : N;
  p.scale = scale;
  p.scale_log2e = scale * fa::kLog2e;
  return p;
}

size_t ws_bytes(long tokens, int Hq, int d) {
  (void)d;
  return round_up((size_t)tokens * Hq * sizeof(float), 256);  // D = rowsum(dO o O)
}

// dropout: threshold round(256 p) in 0 .. 255 (0: nothing is dropped) and the mixed seed
int set_dropout(fa::Problem& p, float p_drop, uint64_t seed) {
  if (!(p_drop >= 0.f) || !(p_drop < 1.f)) return FA_ERR_SHAPE;
  long t = std::lround(256.0 * (double)p_drop);
  if (t > 255) t = 255;
  p.drop_thr = (uint32_t)t;
  p.drop_seed = (uint32_t)seed ^ ((uint32_t)(seed >> 32) * 0x27D4EB2Fu);
  p.drop_rp = 256.f / (256.f - (float)t);
  return FA_OK;
}

// elementwise mask: strides in elements, multiples of 8 (every 16-byte chunk of M aligned)
int set_mask(fa::Problem& p, const void* M, int Nk, long long bs, long long hs, long long rs) {
  if (!M) return FA_ERR_NULL;
  if (!aligned16(M)) return FA_ERR_ALIGN;
  if (bs < 0 || hs < 0 || rs < (((long long)Nk + 7) & ~7LL)) return FA_ERR_SHAPE;
  if (bs % 8 || hs % 8 || rs % 8) return FA_ERR_SHAPE;
  p.mask = (const __bf16*)M;
  p.mask_bs = (long)bs;
  p.mask_hs = (long)hs;
  p.mask_rs = (long)rs;
  return FA_OK;
}

// What an entry point may ask for beyond the plain pass.
struct Options {
  int f16 = 0;                      // element type: 0 bfloat16, 1 IEEE half precision
  bool dropout = false;             // dropout on P with p_drop, seed
  float p_drop = 0.f;
  uint64_t seed = 0;
  bool mask = false;                // elementwise mask M with its three strides
  const void* M = nullptr;
  long long mask_bs = 0, mask_hs = 0, mask_rs = 0;
  bool window = false;              // sliding window (win_left, win_right); a negative bound is no bound
  int win_left = -1, win_right = -1;
  const void* bmask = nullptr;      // block-sparse pattern (with window = true): bytes, two strides, block size
  long long bmask_bs = 0, bmask_hs = 0;
  int block = 0;
  const int32_t* seqlens_k = nullptr;    // key/value cache (split forward only): per-sequence lengths,
  const int32_t* block_table = nullptr;  // page table with its row stride, log2 of the page size
  int page_log2 = 0, table_stride = 0;
  void* dM = nullptr;                    // masked backward: where the gradient of the mask goes, with its strides
  long long dm_bs = 0, dm_hs = 0, dm_rs = 0;
};

Options half_precision(int f16) {
  Options o;
  o.f16 = f16;
  return o;
}
Options of_type(Options o, int f16) {
  o.f16 = f16;
  return o;
}
Options with_dropout(float p_drop, uint64_t seed) {
  Options o;
  o.dropout = true;
  o.p_drop = p_drop;
  o.seed = seed;
  return o;
}
Options with_mask(const void* M, long long bs, long long hs, long long rs) {
  Options o;
  o.mask = true;
  o.M = M;
  o.mask_bs = bs;
  o.mask_hs = hs;
  o.mask_rs = rs;
  return o;
}

Options with_window(int left, int right) {
  Options o;
  o.window = true;
  o.win_left = left < 0 ? -1 : left;
  o.win_right = right < 0 ? -1 : right;
  return o;
}

// block-sparse pattern: block a power of two >= 64; the wavefronts' activity bitmaps hold
// kPatternWords * 64 key blocks (forward, dQ) and row tiles (dK/dV: tiles of 32 rows, one per
// query head of a group)
int set_block_pattern(fa::Problem& p, const Options& o) {
  if (!o.bmask) return FA_ERR_NULL;
  if (o.block < 64 || (o.block & (o.block - 1)) || o.bmask_bs < 0 || o.bmask_hs < 0) return FA_ERR_SHAPE;
  const long words = 64L * fa::kPatternWords;
  if (((long)p.Nk + 63) / 64 > words || (((long)p.N + 31) / 32) * p.G > words) return FA_ERR_UNSUPPORTED;
  p.bmask = (const uint8_t*)o.bmask;
  p.bmask_bs = (long)o.bmask_bs;
  p.bmask_hs = (long)o.bmask_hs;
  p.bmask_cols = (p.Nk + o.block - 1) / o.block;
  p.bmask_log2 = __builtin_ctz((unsigned)o.block);
  return FA_OK;
}

int apply_options(fa::Problem& p, const Options& o) {
  if (o.window) {
    p.win_left = o.win_left;
    p.win_right = o.win_right;
    if (o.block)
      if (int e = set_block_pattern(p, o)) return e;
  }
  if (o.dropout)
    if (int e = set_dropout(p, o.p_drop, o.seed)) return e;
  if (o.mask)
    if (int e = set_mask(p, o.M, p.Nk, o.mask_bs, o.mask_hs, o.mask_rs)) return e;
  return FA_OK;
}

int run_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, const int32_t* cu, int nseq, int N,
            int Nk, long total, int Hq, int Hkv, int d, float scale, int causal, void* stream, int nsplit = 0,
            void* ws = nullptr, const int32_t* cu_k = nullptr, const Options& opt = Options()) {
  fa::FwdArgs a;
  a.nsplit = nsplit;
  a.Opart = (float*)ws;  // [nsplit, tokens, Hq, d], then the partial logsumexps [nsplit, B, Hq, Nq]
  a.Lpart = ws ? (float*)ws + (size_t)nsplit * total * Hq * d : nullptr;
  a.p = make_problem(cu, nseq, N, Nk, Hq, Hkv, d, total, scale, cu_k, opt.f16);
  if (int e = apply_options(a.p, opt)) return e;
  a.seqlens_k = opt.seqlens_k;
  a.block_table = opt.block_table;
  a.page_log2 = opt.page_log2;
  a.table_stride = opt.table_stride;
  a.Q = (const __bf16*)Q;
  a.K = (const __bf16*)K;
  a.V = (const __bf16*)V;
  a.O = (__bf16*)O;
  a.LSE = LSE;
  hipError_t e = fa::launch_fwd(a, d, causal, (hipStream_t)stream);
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    return FA_ERR_LAUNCH;
  }
  return FA_OK;
}

int run_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE, void* dQ,
            void* dK, void* dV, void* ws, const int32_t* cu, int nseq, int N, int Nk, long total, int Hq, int Hkv, int d,
            float scale, int causal, int stages, void* stream, const int32_t* cu_k = nullptr,
            const Options& opt = Options()) {
  fa::BwdArgs a;
  a.p = make_problem(cu, nseq, N, Nk, Hq, Hkv, d, total, scale, cu_k, opt.f16);
  if (int e = apply_options(a.p, opt)) return e;
  a.Q = (const __bf16*)Q;
  a.K = (const __bf16*)K;
  a.V = (const __bf16*)V;
  a.O = (const __bf16*)O;
  a.dO = (const __bf16*)dO;
  a.LSE = LSE;
  a.dQ = (__bf16*)dQ;
  a.dK = (__bf16*)dK;
  a.dV = (__bf16*)dV;
  a.Dvec = (float*)ws;
  a.dM = (__bf16*)opt.dM;
  a.dm_bs = (long)opt.dm_bs;
  a.dm_hs = (long)opt.dm_hs;
  a.dm_rs = (long)opt.dm_rs;
  hipError_t e = fa::launch_bwd(a, d, causal, stages, (hipStream_t)stream);
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    return FA_ERR_LAUNCH;
  }
  return FA_OK;
}

}  // namespace

extern "C" {

int fa_version(void) { return 100; }

const char* fa_status_string(int status) {
  switch (status) {
    case FA_OK: return "ok";
    case FA_ERR_NULL: return "a required pointer is NULL";
    case FA_ERR_SHAPE: return "invalid shape, head grouping, scale or ragged description";
    case FA_ERR_UNSUPPORTED:
      return "unsupported head dimension (multiples of 8 up to 128; dropout, mask and split keys: 64 and 128 only)";
    case FA_ERR_ALIGN: return "a tensor pointer is not 16-byte aligned";
    case FA_ERR_WORKSPACE:
      return "workspace too small (fa_bwd_noalloc: more than FA_NOALLOC_MAX_ROWS (query row, head) pairs)";
    case FA_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    default: return "unknown status";
  }
}

int fa_last_hip_error(void) { return g_last_hip_error; }

int fa_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int N, int d,
           float scale, int causal, void* stream) {
  if (!Q || !K || !V || !O || !LSE) return FA_ERR_NULL;
  if (B <= 0 || N <= 0) return FA_ERR_SHAPE;
  if (int e = check_common(Hq, Hkv, d, scale)) return e;
  if ((long)B * N > 0x7fffffffL) return FA_ERR_SHAPE;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE)) return FA_ERR_ALIGN;
  return run_fwd(Q, K, V, O, LSE, nullptr, B, N, N, (long)B * N, Hq, Hkv, d, scale, causal, stream);
}

size_t fa_bwd_workspace_bytes(int B, int Hq, int Hkv, int N, int d) {
  (void)Hkv;
  if (B <= 0 || Hq <= 0 || N <= 0 || d <= 0) return 0;
  return ws_bytes((long)B * N, Hq, d);
}

int fa_bwd_stages(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                  void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv, int N,
                  int d, float scale, int causal, int stages, void* stream) {
  if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV || !workspace) return FA_ERR_NULL;
  if (B <= 0 || N <= 0) return FA_ERR_SHAPE;
  if (int e = check_common(Hq, Hkv, d, scale)) return e;
  if ((long)B * N > 0x7fffffffL) return FA_ERR_SHAPE;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(dO) || !aligned16(LSE) ||
      !aligned16(dQ) || !aligned16(dK) || !aligned16(dV) || !aligned16(workspace))
    return FA_ERR_ALIGN;
  if (workspace_bytes < ws_bytes((long)B * N, Hq, d)) return FA_ERR_WORKSPACE;
  if (stages <= 0 || (stages & ~7)) return FA_ERR_SHAPE;
  return run_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, nullptr, B, N, N, (long)B * N, Hq, Hkv, d, scale, causal,
                 stages, stream);
}

int fa_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE, void* dQ,
           void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv, int N, int d,
           float scale, int causal, void* stream) {
  return fa_bwd_stages(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, N, d, scale, causal,
                       FA_STAGE_PREP | FA_STAGE_DKDV | FA_STAGE_DQ, stream);
}

int fa_bwd_noalloc(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                   void* dQ, void* dK, void* dV, int B, int Hq, int Hkv, int N, int d, float scale, int causal,
                   void* stream) {
  // sizes first: a problem that does not fit the static array is refused before anything else happens
  if (B > 0 && Hq > 0 && N > 0 && (long long)B * N * Hq > (long long)FA_NOALLOC_MAX_ROWS) return FA_ERR_WORKSPACE;
  float* ws = nullptr;
  if (int e = scratch_on_current_device(&ws, &g_last_hip_error)) return e;
  return fa_bwd_stages(Q, K, V, O, dO, LSE, dQ, dK, dV, ws, sizeof(float) * (size_t)FA_NOALLOC_MAX_ROWS, B, Hq, Hkv, N,
                       d, scale, causal, FA_STAGE_PREP | FA_STAGE_DKDV | FA_STAGE_DQ, stream);
}

static int check_varlen(const int32_t* cu, int nseq, int total_tokens, int max_seqlen) {
  if (!cu) return FA_ERR_NULL;
  if (nseq <= 0 || total_tokens <= 0 || max_seqlen <= 0) return FA_ERR_SHAPE;
  if (max_seqlen > total_tokens) return FA_ERR_SHAPE;
  if ((long)max_seqlen * nseq < (long)total_tokens) return FA_ERR_SHAPE;  // lengths cannot add up
  return FA_OK;
}

static int varlen_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, const int32_t* cu_seqlens,
                      int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv, int d, float scale, int causal,
                      void* stream, const Options& opt) {
  if (!Q || !K || !V || !O || !LSE) return FA_ERR_NULL;
  if (int e = check_varlen(cu_seqlens, nseq, total_tokens, max_seqlen)) return e;
  if (int e = check_common(Hq, Hkv, d, scale, !(opt.dropout || opt.window))) return e;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE)) return FA_ERR_ALIGN;
  return run_fwd(Q, K, V, O, LSE, cu_seqlens, nseq, max_seqlen, max_seqlen, total_tokens, Hq, Hkv, d, scale, causal,
                 stream, 0, nullptr, nullptr, opt);
}

static int varlen_fwd_any(int f16, const void* Q, const void* K, const void* V, void* O, float* LSE,
                          const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv,
                          int d, float scale, int causal, void* stream) {
  return varlen_fwd(Q, K, V, O, LSE, cu_seqlens, nseq, total_tokens, max_seqlen, Hq, Hkv, d, scale, causal, stream,
                    half_precision(f16));
}

int fa_varlen_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, const int32_t* cu_seqlens,
                  int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv, int d, float scale, int causal,
                  void* stream) {
  return varlen_fwd_any(0, Q, K, V, O, LSE, cu_seqlens, nseq, total_tokens, max_seqlen, Hq, Hkv, d, scale, causal,
                        stream);
}

int fa_varlen_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE, const int32_t* cu_seqlens,
                      int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv, int d, float scale, int causal,
                      void* stream) {
  return varlen_fwd_any(1, Q, K, V, O, LSE, cu_seqlens, nseq, total_tokens, max_seqlen, Hq, Hkv, d, scale, causal,
                        stream);
}

static int varlen_dropout_fwd_any(int f16, const void* Q, const void* K, const void* V, void* O, float* LSE,
                                  const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq,
                                  int Hkv, int d, float scale, int causal, float p_drop, uint64_t seed,
                                  void* stream) {
  return varlen_fwd(Q, K, V, O, LSE, cu_seqlens, nseq, total_tokens, max_seqlen, Hq, Hkv, d, scale, causal, stream,
                    of_type(with_dropout(p_drop, seed), f16));
}

int fa_varlen_dropout_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, const int32_t* cu_seqlens,
                          int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv, int d, float scale, int causal,
                          float p_drop, uint64_t seed, void* stream) {
  return varlen_dropout_fwd_any(0, Q, K, V, O, LSE, cu_seqlens, nseq, total_tokens, max_seqlen, Hq, Hkv, d, scale,
                                causal, p_drop, seed, stream);
}

int fa_varlen_dropout_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                              const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv,
                              int d, float scale, int causal, float p_drop, uint64_t seed, void* stream) {
  return varlen_dropout_fwd_any(1, Q, K, V, O, LSE, cu_seqlens, nseq, total_tokens, max_seqlen, Hq, Hkv, d, scale,
                                causal, p_drop, seed, stream);
}

size_t fa_varlen_bwd_workspace_bytes(int total_tokens, int Hq, int Hkv, int d) {
  (void)Hkv;
  if (total_tokens <= 0 || Hq <= 0 || d <= 0) return 0;
  return ws_bytes(total_tokens, Hq, d);
}

static int varlen_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                      void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                      const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv, int d,
                      float scale, int causal, void* stream, const Options& opt) {
  if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV || !workspace) return FA_ERR_NULL;
  if (int e = check_varlen(cu_seqlens, nseq, total_tokens, max_seqlen)) return e;
  if (int e = check_common(Hq, Hkv, d, scale, !(opt.dropout || opt.window))) return e;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(dO) || !aligned16(LSE) ||
      !aligned16(dQ) || !aligned16(dK) || !aligned16(dV) || !aligned16(workspace))
    return FA_ERR_ALIGN;
  if (workspace_bytes < ws_bytes(total_tokens, Hq, d)) return FA_ERR_WORKSPACE;
  return run_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, cu_seqlens, nseq, max_seqlen, max_seqlen, total_tokens, Hq,
                 Hkv, d, scale, causal, 7, stream, nullptr, opt);
}

static int varlen_bwd_any(int f16, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                          const float* LSE, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                          const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv,
                          int d, float scale, int causal, void* stream) {
  return varlen_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens, nseq, total_tokens,
                    max_seqlen, Hq, Hkv, d, scale, causal, stream, half_precision(f16));
}

int fa_varlen_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                  void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, const int32_t* cu_seqlens,
                  int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv, int d, float scale, int causal,
                  void* stream) {
  return varlen_bwd_any(0, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens, nseq,
                        total_tokens, max_seqlen, Hq, Hkv, d, scale, causal, stream);
}

int fa_varlen_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                      void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                      const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv, int d,
                      float scale, int causal, void* stream) {
  return varlen_bwd_any(1, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens, nseq,
                        total_tokens, max_seqlen, Hq, Hkv, d, scale, causal, stream);
}

static int varlen_dropout_bwd_any(int f16, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                                  const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                                  size_t workspace_bytes, const int32_t* cu_seqlens, int nseq, int total_tokens,
                                  int max_seqlen, int Hq, int Hkv, int d, float scale, int causal, float p_drop,
                                  uint64_t seed, void* stream) {
  return varlen_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens, nseq, total_tokens,
                    max_seqlen, Hq, Hkv, d, scale, causal, stream, of_type(with_dropout(p_drop, seed), f16));
}

int fa_varlen_dropout_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                          const float* LSE, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                          const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv,
                          int d, float scale, int causal, float p_drop, uint64_t seed, void* stream) {
  return varlen_dropout_bwd_any(0, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens, nseq,
                                total_tokens, max_seqlen, Hq, Hkv, d, scale, causal, p_drop, seed, stream);
}

int fa_varlen_dropout_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                              const float* LSE, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                              const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv,
                              int d, float scale, int causal, float p_drop, uint64_t seed, void* stream) {
  return varlen_dropout_bwd_any(1, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens, nseq,
                                total_tokens, max_seqlen, Hq, Hkv, d, scale, causal, p_drop, seed, stream);
}

static int check_cross(int B, int Nq, int Nk, int causal) {
  if (B <= 0 || Nq <= 0 || Nk <= 0) return FA_ERR_SHAPE;
  if (causal && Nq > Nk) return FA_ERR_SHAPE;  // some query would see no key
  if ((long)B * Nq > 0x7fffffffL || (long)B * Nk > 0x7fffffffL) return FA_ERR_SHAPE;
  return FA_OK;
}

// Dense entry points with two lengths: the plain ones, half precision, dropout and mask differ
// only in the options.
// (`rule`: the causal rule is in force although `causal` is 0, because a window instantiation applies it)
static int cross_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int Nq,
                     int Nk, int d, float scale, int causal, void* stream, const Options& opt, int rule = 0) {
  if (!Q || !K || !V || !O || !LSE) return FA_ERR_NULL;
  if (int e = check_cross(B, Nq, Nk, causal || rule)) return e;
  if (int e = check_common(Hq, Hkv, d, scale, !(opt.dropout || opt.mask || opt.window))) return e;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE)) return FA_ERR_ALIGN;
  return run_fwd(Q, K, V, O, LSE, nullptr, B, Nq, Nk, (long)B * Nq, Hq, Hkv, d, scale, causal, stream, 0, nullptr,
                 nullptr, opt);
}

static int cross_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                     void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv,
                     int Nq, int Nk, int d, float scale, int causal, void* stream, const Options& opt, int rule = 0) {
  if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV || !workspace) return FA_ERR_NULL;
  if (int e = check_cross(B, Nq, Nk, causal || rule)) return e;
  if (int e = check_common(Hq, Hkv, d, scale, !(opt.dropout || opt.mask || opt.window))) return e;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(dO) || !aligned16(LSE) ||
      !aligned16(dQ) || !aligned16(dK) || !aligned16(dV) || !aligned16(workspace))
    return FA_ERR_ALIGN;
  if (workspace_bytes < ws_bytes((long)B * Nq, Hq, d)) return FA_ERR_WORKSPACE;
  return run_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, nullptr, B, Nq, Nk, (long)B * Nq, Hq, Hkv, d, scale,
                 causal, FA_STAGE_PREP | FA_STAGE_DKDV | FA_STAGE_DQ, stream, nullptr, opt);
}

int fa_cross_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int Nq,
                 int Nk, int d, float scale, int causal, void* stream) {
  return cross_fwd(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, stream, half_precision(0));
}

int fa_cross_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int Nq,
                     int Nk, int d, float scale, int causal, void* stream) {
  return cross_fwd(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, stream, half_precision(1));
}

size_t fa_cross_bwd_workspace_bytes(int B, int Hq, int Hkv, int Nq, int Nk, int d) {
  (void)Hkv;
  if (B <= 0 || Hq <= 0 || Nq <= 0 || Nk <= 0 || d <= 0) return 0;
  return ws_bytes((long)B * Nq, Hq, d);
}

int fa_cross_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                 void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv,
                 int Nq, int Nk, int d, float scale, int causal, void* stream) {
  return cross_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal,
                   stream, half_precision(0));
}

int fa_cross_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                     void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv,
                     int Nq, int Nk, int d, float scale, int causal, void* stream) {
  return cross_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal,
                   stream, half_precision(1));
}

static int dropout_fwd_any(int f16, const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq,
                           int Hkv, int Nq, int Nk, int d, float scale, int causal, float p_drop, uint64_t seed,
                           void* stream) {
  return cross_fwd(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, stream,
                   of_type(with_dropout(p_drop, seed), f16));
}

int fa_dropout_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int Nq,
                   int Nk, int d, float scale, int causal, float p_drop, uint64_t seed, void* stream) {
  return dropout_fwd_any(0, Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, p_drop, seed, stream);
}

int fa_dropout_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv,
                       int Nq, int Nk, int d, float scale, int causal, float p_drop, uint64_t seed, void* stream) {
  return dropout_fwd_any(1, Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, p_drop, seed, stream);
}

static int dropout_bwd_any(int f16, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                           const float* LSE, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                           int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal, float p_drop,
                           uint64_t seed, void* stream) {
  return cross_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal,
                   stream, of_type(with_dropout(p_drop, seed), f16));
}

int fa_dropout_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                   void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv,
                   int Nq, int Nk, int d, float scale, int causal, float p_drop, uint64_t seed, void* stream) {
  return dropout_bwd_any(0, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale,
                         causal, p_drop, seed, stream);
}

int fa_dropout_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                       void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv,
                       int Nq, int Nk, int d, float scale, int causal, float p_drop, uint64_t seed, void* stream) {
  return dropout_bwd_any(1, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale,
                         causal, p_drop, seed, stream);
}

static int mask_fwd_any(int f16, const void* Q, const void* K, const void* V, const void* M, void* O, float* LSE,
                        int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                        long long mask_batch_stride, long long mask_head_stride, long long mask_row_stride,
                        void* stream) {
  return cross_fwd(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, stream,
                   of_type(with_mask(M, mask_batch_stride, mask_head_stride, mask_row_stride), f16));
}

int fa_mask_fwd(const void* Q, const void* K, const void* V, const void* M, void* O, float* LSE, int B, int Hq,
                int Hkv, int Nq, int Nk, int d, float scale, int causal, long long mask_batch_stride,
                long long mask_head_stride, long long mask_row_stride, void* stream) {
  return mask_fwd_any(0, Q, K, V, M, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, mask_batch_stride, mask_head_stride,
                      mask_row_stride, stream);
}

int fa_mask_fwd_f16(const void* Q, const void* K, const void* V, const void* M, void* O, float* LSE, int B, int Hq,
                    int Hkv, int Nq, int Nk, int d, float scale, int causal, long long mask_batch_stride,
                    long long mask_head_stride, long long mask_row_stride, void* stream) {
  return mask_fwd_any(1, Q, K, V, M, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, mask_batch_stride, mask_head_stride,
                      mask_row_stride, stream);
}

static int mask_bwd_any(int f16, const void* Q, const void* K, const void* V, const void* M, const void* O,
                        const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                        size_t workspace_bytes, int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                        long long mask_batch_stride, long long mask_head_stride, long long mask_row_stride,
                        void* stream) {
  return cross_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal,
                   stream, of_type(with_mask(M, mask_batch_stride, mask_head_stride, mask_row_stride), f16));
}

int fa_mask_bwd(const void* Q, const void* K, const void* V, const void* M, const void* O, const void* dO,
                const float* LSE, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq,
                int Hkv, int Nq, int Nk, int d, float scale, int causal, long long mask_batch_stride,
                long long mask_head_stride, long long mask_row_stride, void* stream) {
  return mask_bwd_any(0, Q, K, V, M, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale,
                      causal, mask_batch_stride, mask_head_stride, mask_row_stride, stream);
}

int fa_mask_bwd_f16(const void* Q, const void* K, const void* V, const void* M, const void* O, const void* dO,
                    const float* LSE, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B,
                    int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal, long long mask_batch_stride,
                    long long mask_head_stride, long long mask_row_stride, void* stream) {
  return mask_bwd_any(1, Q, K, V, M, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale,
                      causal, mask_batch_stride, mask_head_stride, mask_row_stride, stream);
}

static int mask_bwd_dmask_any(int f16, const void* Q, const void* K, const void* V, const void* M, const void* O,
                              const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* dM, void* workspace,
                              size_t workspace_bytes, int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale,
                              int causal, long long mask_batch_stride, long long mask_head_stride,
                              long long mask_row_stride, long long dmask_batch_stride, long long dmask_head_stride,
                              long long dmask_row_stride, void* stream) {
  if (!dM) return FA_ERR_NULL;
  if (!aligned16(dM)) return FA_ERR_ALIGN;
  // every (sequence, head) has rows of its own in dM: strides as for M, none of them zero
  if (dmask_row_stride < (((long long)Nk + 7) & ~7LL) || dmask_row_stride % 8 || dmask_head_stride % 8 ||
      dmask_batch_stride % 8 || dmask_head_stride < dmask_row_stride * Nq ||
      dmask_batch_stride < dmask_head_stride * Hq)
    return FA_ERR_SHAPE;
  Options opt = of_type(with_mask(M, mask_batch_stride, mask_head_stride, mask_row_stride), f16);
  opt.dM = dM;
  opt.dm_bs = dmask_batch_stride;
  opt.dm_hs = dmask_head_stride;
  opt.dm_rs = dmask_row_stride;
  return cross_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal,
                   stream, opt);
}

int fa_mask_bwd_dmask(const void* Q, const void* K, const void* V, const void* M, const void* O, const void* dO,
                      const float* LSE, void* dQ, void* dK, void* dV, void* dM, void* workspace, size_t workspace_bytes,
                      int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                      long long mask_batch_stride, long long mask_head_stride, long long mask_row_stride,
                      long long dmask_batch_stride, long long dmask_head_stride, long long dmask_row_stride,
                      void* stream) {
  return mask_bwd_dmask_any(0, Q, K, V, M, O, dO, LSE, dQ, dK, dV, dM, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d,
                            scale, causal, mask_batch_stride, mask_head_stride, mask_row_stride, dmask_batch_stride,
                            dmask_head_stride, dmask_row_stride, stream);
}

int fa_mask_bwd_dmask_f16(const void* Q, const void* K, const void* V, const void* M, const void* O, const void* dO,
                          const float* LSE, void* dQ, void* dK, void* dV, void* dM, void* workspace,
                          size_t workspace_bytes, int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                          long long mask_batch_stride, long long mask_head_stride, long long mask_row_stride,
                          long long dmask_batch_stride, long long dmask_head_stride, long long dmask_row_stride,
                          void* stream) {
  return mask_bwd_dmask_any(1, Q, K, V, M, O, dO, LSE, dQ, dK, dV, dM, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d,
                            scale, causal, mask_batch_stride, mask_head_stride, mask_row_stride, dmask_batch_stride,
                            dmask_head_stride, dmask_row_stride, stream);
}

// Sliding window. Without any bound this is plain attention and with win_right = 0 alone the
// causal rule: both go to the kernels built for them. Otherwise the window instantiations run.
static int window_route(int Nq, int Nk, int& left, int& right, int& causal) {
  if (Nq > Nk) return FA_ERR_SHAPE;  // some query would stand before the first key
  if (left < 0) left = -1;
  if (right < 0) right = -1;
  if (left >= Nk) left = -1;    // a bound no row can reach is no bound
  if (right >= Nk) right = -1;
  causal = left < 0 && right == 0;
  if (causal) right = -1;
  return FA_OK;
}

static int local_fwd_any(int f16, const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq,
                         int Hkv, int Nq, int Nk, int d, float scale, int window_left, int window_right,
                         void* stream) {
  int causal = 0;
  if (B > 0 && Nq > 0 && Nk > 0)
    if (int e = window_route(Nq, Nk, window_left, window_right, causal)) return e;
  const bool none = window_left < 0 && window_right < 0;
  return cross_fwd(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, stream,
                   none ? half_precision(f16) : of_type(with_window(window_left, window_right), f16));
}

int fa_local_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int Nq,
                 int Nk, int d, float scale, int window_left, int window_right, void* stream) {
  return local_fwd_any(0, Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, window_left, window_right, stream);
}

int fa_local_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq, int Hkv, int Nq,
                     int Nk, int d, float scale, int window_left, int window_right, void* stream) {
  return local_fwd_any(1, Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, window_left, window_right, stream);
}

static int local_bwd_any(int f16, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                         const float* LSE, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                         int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int window_left, int window_right,
                         void* stream) {
  int causal = 0;
  if (B > 0 && Nq > 0 && Nk > 0)
    if (int e = window_route(Nq, Nk, window_left, window_right, causal)) return e;
  const bool none = window_left < 0 && window_right < 0;
  return cross_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal,
                   stream, none ? half_precision(f16) : of_type(with_window(window_left, window_right), f16));
}

int fa_local_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                 void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv, int Nq,
                 int Nk, int d, float scale, int window_left, int window_right, void* stream) {
  return local_bwd_any(0, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale,
                       window_left, window_right, stream);
}

int fa_local_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                     void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv,
                     int Nq, int Nk, int d, float scale, int window_left, int window_right, void* stream) {
  return local_bwd_any(1, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale,
                       window_left, window_right, stream);
}

static Options with_block_pattern(const void* block_mask, int block, long long bs, long long hs, int causal) {
  Options o = with_window(-1, causal ? 0 : -1);  // the causal rule is the window (none, 0)
  o.bmask = block_mask;
  o.bmask_bs = bs;
  o.bmask_hs = hs;
  o.block = block ? block : -1;  // (0 would read as "no pattern")
  return o;
}

static int blocksparse_fwd_any(int f16, const void* Q, const void* K, const void* V, const void* block_mask, void* O,
                               float* LSE, int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                               int block, long long mask_batch_stride, long long mask_head_stride, void* stream) {
  if (!block_mask) return FA_ERR_NULL;
  return cross_fwd(Q, K, V, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, 0, stream,
                   of_type(with_block_pattern(block_mask, block, mask_batch_stride, mask_head_stride, causal), f16),
                   causal);
}

int fa_blocksparse_fwd(const void* Q, const void* K, const void* V, const void* block_mask, void* O, float* LSE, int B,
                       int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal, int block,
                       long long mask_batch_stride, long long mask_head_stride, void* stream) {
  return blocksparse_fwd_any(0, Q, K, V, block_mask, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, block,
                             mask_batch_stride, mask_head_stride, stream);
}

int fa_blocksparse_fwd_f16(const void* Q, const void* K, const void* V, const void* block_mask, void* O, float* LSE,
                           int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal, int block,
                           long long mask_batch_stride, long long mask_head_stride, void* stream) {
  return blocksparse_fwd_any(1, Q, K, V, block_mask, O, LSE, B, Hq, Hkv, Nq, Nk, d, scale, causal, block,
                             mask_batch_stride, mask_head_stride, stream);
}

static int blocksparse_bwd_any(int f16, const void* Q, const void* K, const void* V, const void* block_mask,
                               const void* O, const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                               void* workspace, size_t workspace_bytes, int B, int Hq, int Hkv, int Nq, int Nk, int d,
                               float scale, int causal, int block, long long mask_batch_stride,
                               long long mask_head_stride, void* stream) {
  if (!block_mask) return FA_ERR_NULL;
  return cross_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale, 0, stream,
                   of_type(with_block_pattern(block_mask, block, mask_batch_stride, mask_head_stride, causal), f16),
                   causal);
}

int fa_blocksparse_bwd(const void* Q, const void* K, const void* V, const void* block_mask, const void* O,
                       const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                       size_t workspace_bytes, int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                       int block, long long mask_batch_stride, long long mask_head_stride, void* stream) {
  return blocksparse_bwd_any(0, Q, K, V, block_mask, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv,
                             Nq, Nk, d, scale, causal, block, mask_batch_stride, mask_head_stride, stream);
}

int fa_blocksparse_bwd_f16(const void* Q, const void* K, const void* V, const void* block_mask, const void* O,
                           const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                           size_t workspace_bytes, int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale,
                           int causal, int block, long long mask_batch_stride, long long mask_head_stride,
                           void* stream) {
  return blocksparse_bwd_any(1, Q, K, V, block_mask, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, Hq, Hkv,
                             Nq, Nk, d, scale, causal, block, mask_batch_stride, mask_head_stride, stream);
}

int fa_fp8_fwd(const void* Q8, const void* K8, const void* Vt8, void* O, float* LSE, int B, int Hq, int Hkv, int Nq,
               int Nk, int d, long long vt_stride, float scale, float descale_q, float descale_k, float descale_v,
               int causal, void* stream) {
  if (!Q8 || !K8 || !Vt8 || !O || !LSE) return FA_ERR_NULL;
  if (int e = check_cross(B, Nq, Nk, causal)) return e;
  if (int e = check_common(Hq, Hkv, d, scale, false)) return e;
  for (float ds : {descale_q, descale_k, descale_v})
    if (!(ds > 0.f) || !std::isfinite(ds)) return FA_ERR_SHAPE;
  if (vt_stride % 64 != 0 || vt_stride < ((long long)Nk + 63) / 64 * 64) return FA_ERR_SHAPE;
  if (!aligned16(Q8) || !aligned16(K8) || !aligned16(Vt8) || !aligned16(O) || !aligned16(LSE)) return FA_ERR_ALIGN;
  fa::Fp8Args a;
  a.p = make_problem(nullptr, B, Nq, Nk, Hq, Hkv, d, (long)B * Nq, scale * descale_q * descale_k);
  a.Q = Q8;
  a.K = K8;
  a.Vt = Vt8;
  a.O = (__bf16*)O;
  a.LSE = LSE;
  a.vt_stride = (long)vt_stride;
  a.descale_v = descale_v;
  hipError_t e = fa::launch_fwd_fp8(a, d, causal, (hipStream_t)stream);
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    return FA_ERR_LAUNCH;
  }
  return FA_OK;
}

// Sliding window over a packed ragged batch: the routing of fa_local_fwd with the longest
// sequence standing for both lengths (a bound that reaches past it binds nowhere).
static int varlen_local_fwd_any(int f16, const void* Q, const void* K, const void* V, void* O, float* LSE,
                                const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq,
                                int Hkv, int d, float scale, int window_left, int window_right, void* stream) {
  int causal = 0;
  if (max_seqlen > 0)
    if (int e = window_route(max_seqlen, max_seqlen, window_left, window_right, causal)) return e;
  const bool none = window_left < 0 && window_right < 0;
  return varlen_fwd(Q, K, V, O, LSE, cu_seqlens, nseq, total_tokens, max_seqlen, Hq, Hkv, d, scale, causal, stream,
                    none ? half_precision(f16) : of_type(with_window(window_left, window_right), f16));
}

int fa_varlen_local_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, const int32_t* cu_seqlens,
                        int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv, int d, float scale,
                        int window_left, int window_right, void* stream) {
  return varlen_local_fwd_any(0, Q, K, V, O, LSE, cu_seqlens, nseq, total_tokens, max_seqlen, Hq, Hkv, d, scale,
                              window_left, window_right, stream);
}

int fa_varlen_local_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                            const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv,
                            int d, float scale, int window_left, int window_right, void* stream) {
  return varlen_local_fwd_any(1, Q, K, V, O, LSE, cu_seqlens, nseq, total_tokens, max_seqlen, Hq, Hkv, d, scale,
                              window_left, window_right, stream);
}

static int varlen_local_bwd_any(int f16, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                                const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                                size_t workspace_bytes, const int32_t* cu_seqlens, int nseq, int total_tokens,
                                int max_seqlen, int Hq, int Hkv, int d, float scale, int window_left,
                                int window_right, void* stream) {
  int causal = 0;
  if (max_seqlen > 0)
    if (int e = window_route(max_seqlen, max_seqlen, window_left, window_right, causal)) return e;
  const bool none = window_left < 0 && window_right < 0;
  return varlen_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens, nseq, total_tokens,
                    max_seqlen, Hq, Hkv, d, scale, causal, stream,
                    none ? half_precision(f16) : of_type(with_window(window_left, window_right), f16));
}

int fa_varlen_local_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                        void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                        const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv, int d,
                        float scale, int window_left, int window_right, void* stream) {
  return varlen_local_bwd_any(0, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens, nseq,
                              total_tokens, max_seqlen, Hq, Hkv, d, scale, window_left, window_right, stream);
}

int fa_varlen_local_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                            const float* LSE, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                            const int32_t* cu_seqlens, int nseq, int total_tokens, int max_seqlen, int Hq, int Hkv,
                            int d, float scale, int window_left, int window_right, void* stream) {
  return varlen_local_bwd_any(1, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens, nseq,
                              total_tokens, max_seqlen, Hq, Hkv, d, scale, window_left, window_right, stream);
}

static int check_varlen_cross(const int32_t* cu_q, const int32_t* cu_k, int nseq, int total_q, int total_k, int max_q,
                              int max_k) {
  if (int e = check_varlen(cu_q, nseq, total_q, max_q)) return e;
  return check_varlen(cu_k, nseq, total_k, max_k);
}

static int varlen_cross_fwd_any(int f16, const void* Q, const void* K, const void* V, void* O, float* LSE,
                                const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int nseq, int total_q,
                                int total_k, int max_seqlen_q, int max_seqlen_k, int Hq, int Hkv, int d, float scale,
                                int causal, void* stream) {
  if (!Q || !K || !V || !O || !LSE) return FA_ERR_NULL;
  if (int e = check_varlen_cross(cu_seqlens_q, cu_seqlens_k, nseq, total_q, total_k, max_seqlen_q, max_seqlen_k)) return e;
  if (int e = check_common(Hq, Hkv, d, scale)) return e;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE)) return FA_ERR_ALIGN;
  return run_fwd(Q, K, V, O, LSE, cu_seqlens_q, nseq, max_seqlen_q, max_seqlen_k, total_q, Hq, Hkv, d, scale, causal,
                 stream, 0, nullptr, cu_seqlens_k, half_precision(f16));
}

int fa_varlen_cross_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, const int32_t* cu_seqlens_q,
                        const int32_t* cu_seqlens_k, int nseq, int total_q, int total_k, int max_seqlen_q,
                        int max_seqlen_k, int Hq, int Hkv, int d, float scale, int causal, void* stream) {
  return varlen_cross_fwd_any(0, Q, K, V, O, LSE, cu_seqlens_q, cu_seqlens_k, nseq, total_q, total_k, max_seqlen_q,
                              max_seqlen_k, Hq, Hkv, d, scale, causal, stream);
}

int fa_varlen_cross_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE,
                            const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int nseq, int total_q,
                            int total_k, int max_seqlen_q, int max_seqlen_k, int Hq, int Hkv, int d, float scale,
                            int causal, void* stream) {
  return varlen_cross_fwd_any(1, Q, K, V, O, LSE, cu_seqlens_q, cu_seqlens_k, nseq, total_q, total_k, max_seqlen_q,
                              max_seqlen_k, Hq, Hkv, d, scale, causal, stream);
}

static int varlen_cross_bwd_any(int f16, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                                const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                                size_t workspace_bytes, const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k,
                                int nseq, int total_q, int total_k, int max_seqlen_q, int max_seqlen_k, int Hq,
                                int Hkv, int d, float scale, int causal, void* stream) {
  if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV || !workspace) return FA_ERR_NULL;
  if (int e = check_varlen_cross(cu_seqlens_q, cu_seqlens_k, nseq, total_q, total_k, max_seqlen_q, max_seqlen_k)) return e;
  if (int e = check_common(Hq, Hkv, d, scale)) return e;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(dO) || !aligned16(LSE) ||
      !aligned16(dQ) || !aligned16(dK) || !aligned16(dV) || !aligned16(workspace))
    return FA_ERR_ALIGN;
  if (workspace_bytes < ws_bytes(total_q, Hq, d)) return FA_ERR_WORKSPACE;
  return run_bwd(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, cu_seqlens_q, nseq, max_seqlen_q, max_seqlen_k, total_q,
                 Hq, Hkv, d, scale, causal, 7, stream, cu_seqlens_k, half_precision(f16));
}

int fa_varlen_cross_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                        void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                        const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int nseq, int total_q, int total_k,
                        int max_seqlen_q, int max_seqlen_k, int Hq, int Hkv, int d, float scale, int causal,
                        void* stream) {
  return varlen_cross_bwd_any(0, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens_q,
                              cu_seqlens_k, nseq, total_q, total_k, max_seqlen_q, max_seqlen_k, Hq, Hkv, d, scale,
                              causal, stream);
}

int fa_varlen_cross_bwd_f16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                            const float* LSE, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                            const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int nseq, int total_q,
                            int total_k, int max_seqlen_q, int max_seqlen_k, int Hq, int Hkv, int d, float scale,
                            int causal, void* stream) {
  return varlen_cross_bwd_any(1, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, cu_seqlens_q,
                              cu_seqlens_k, nseq, total_q, total_k, max_seqlen_q, max_seqlen_k, Hq, Hkv, d, scale,
                              causal, stream);
}

size_t fa_splitkv_fwd_workspace_bytes(int B, int Hq, int Nq, int d, int num_splits) {
  if (B <= 0 || Hq <= 0 || Nq <= 0 || d <= 0 || num_splits <= 0) return 0;
  return round_up((size_t)num_splits * B * Nq * Hq * (d + 1) * sizeof(float), 256);
}

static int splitkv_fwd_any(int f16, const void* Q, const void* K, const void* V, void* O, float* LSE, void* workspace,
                           size_t workspace_bytes, int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale,
                           int causal, int num_splits, void* stream) {
  if (!Q || !K || !V || !O || !LSE || !workspace) return FA_ERR_NULL;
  if (int e = check_cross(B, Nq, Nk, causal)) return e;
  if (int e = check_common(Hq, Hkv, d, scale, false)) return e;
  if (num_splits < 1 || num_splits > FA_SPLITKV_MAX_SPLITS) return FA_ERR_SHAPE;
  if ((long)Nq * (Hq / Hkv) > 0x7fffffffL) return FA_ERR_SHAPE;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE) || !aligned16(workspace))
    return FA_ERR_ALIGN;
  if (workspace_bytes < fa_splitkv_fwd_workspace_bytes(B, Hq, Nq, d, num_splits)) return FA_ERR_WORKSPACE;
  return run_fwd(Q, K, V, O, LSE, nullptr, B, Nq, Nk, (long)B * Nq, Hq, Hkv, d, scale, causal, stream, num_splits,
                 workspace, nullptr, half_precision(f16));
}

int fa_splitkv_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, void* workspace,
                   size_t workspace_bytes, int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                   int num_splits, void* stream) {
  return splitkv_fwd_any(0, Q, K, V, O, LSE, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal,
                         num_splits, stream);
}

int fa_splitkv_fwd_f16(const void* Q, const void* K, const void* V, void* O, float* LSE, void* workspace,
                       size_t workspace_bytes, int B, int Hq, int Hkv, int Nq, int Nk, int d, float scale, int causal,
                       int num_splits, void* stream) {
  return splitkv_fwd_any(1, Q, K, V, O, LSE, workspace, workspace_bytes, B, Hq, Hkv, Nq, Nk, d, scale, causal,
                         num_splits, stream);
}

static int kvcache_fwd_any(int f16, const void* Q, const void* Kcache, const void* Vcache, const int32_t* seqlens_k,
                           const int32_t* block_table, void* O, float* LSE, void* workspace, size_t workspace_bytes,
                           int B, int Hq, int Hkv, int Nq, int Nk, int d, int page_size, int pages_per_seq,
                           float scale, int causal, int num_splits, void* stream) {
  if (!Q || !Kcache || !Vcache || !O || !LSE || !workspace) return FA_ERR_NULL;
  if (int e = check_cross(B, Nq, Nk, causal)) return e;
  if (int e = check_common(Hq, Hkv, d, scale, false)) return e;
  if (num_splits < 1 || num_splits > FA_SPLITKV_MAX_SPLITS) return FA_ERR_SHAPE;
  if ((long)Nq * (Hq / Hkv) > 0x7fffffffL) return FA_ERR_SHAPE;
  Options opt = half_precision(f16);
  opt.seqlens_k = seqlens_k;
  if (block_table) {
    if (page_size < 64 || (page_size & (page_size - 1))) return FA_ERR_UNSUPPORTED;  // whole blocks of 64 keys per page
    if (pages_per_seq < 1 || (long)pages_per_seq * page_size < Nk) return FA_ERR_SHAPE;
    opt.block_table = block_table;
    opt.page_log2 = __builtin_ctz((unsigned)page_size);
    opt.table_stride = pages_per_seq;
  }
  if (!aligned16(Q) || !aligned16(Kcache) || !aligned16(Vcache) || !aligned16(O) || !aligned16(LSE) ||
      !aligned16(workspace) || (reinterpret_cast<uintptr_t>(seqlens_k) & 3u) ||
      (reinterpret_cast<uintptr_t>(block_table) & 3u))
    return FA_ERR_ALIGN;
  if (workspace_bytes < fa_splitkv_fwd_workspace_bytes(B, Hq, Nq, d, num_splits)) return FA_ERR_WORKSPACE;
  return run_fwd(Q, Kcache, Vcache, O, LSE, nullptr, B, Nq, Nk, (long)B * Nq, Hq, Hkv, d, scale, causal, stream,
                 num_splits, workspace, nullptr, opt);
}

int fa_kvcache_fwd(const void* Q, const void* Kcache, const void* Vcache, const int32_t* seqlens_k,
                   const int32_t* block_table, void* O, float* LSE, void* workspace, size_t workspace_bytes, int B,
                   int Hq, int Hkv, int Nq, int Nk, int d, int page_size, int pages_per_seq, float scale, int causal,
                   int num_splits, void* stream) {
  return kvcache_fwd_any(0, Q, Kcache, Vcache, seqlens_k, block_table, O, LSE, workspace, workspace_bytes, B, Hq, Hkv,
                         Nq, Nk, d, page_size, pages_per_seq, scale, causal, num_splits, stream);
}

int fa_kvcache_fwd_f16(const void* Q, const void* Kcache, const void* Vcache, const int32_t* seqlens_k,
                       const int32_t* block_table, void* O, float* LSE, void* workspace, size_t workspace_bytes,
                       int B, int Hq, int Hkv, int Nq, int Nk, int d, int page_size, int pages_per_seq, float scale,
                       int causal, int num_splits, void* stream) {
  return kvcache_fwd_any(1, Q, Kcache, Vcache, seqlens_k, block_table, O, LSE, workspace, workspace_bytes, B, Hq, Hkv,
                         Nq, Nk, d, page_size, pages_per_seq, scale, causal, num_splits, stream);
}

size_t fa_mfma_probe_scratch_bytes(void) { return 16 + (size_t)256 * 512 * sizeof(float); }

int fa_mfma_probe(int iters, int random_operands, void* scratch, void* stream) {
  if (!scratch) return FA_ERR_NULL;
  if ((uintptr_t)scratch % 16 != 0) return FA_ERR_ALIGN;
  if (iters < 1) return FA_ERR_SHAPE;
  hipError_t e = fa::launch_mfma_probe((float*)((char*)scratch + 16), (long long*)scratch, 256, iters,
                                       random_operands, (hipStream_t)stream);
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    return FA_ERR_LAUNCH;
  }
  return FA_OK;
}

}  // extern "C"
