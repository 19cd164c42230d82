// Backward pass of exact attention for gfx950 (Algorithm 2 of the paper).
//
// Three launches on the caller's stream:
//   1. prep:    D = rowsum(dO o O) (Algorithm 2, line 4) and dQ accumulator := 0 (line 3)
//   2. main:    one workgroup per block of BC = 128 keys of one (sequence, key/value
//               head) (section 3.2 "Backward pass"); it loops over the query heads
//               that share the key/value head and over the row blocks i, recomputes
//               P from the saved logsumexp (line 11), keeps dK_j, dV_j in MFMA
//               accumulators for the whole loop and adds its dQ_i contributions to a
//               float32 buffer with atomic adds
//   3. convert: dQ = bf16(scale * accumulator)
//
// Lane layout of the main kernel: each of the 4 wavefronts owns 32 keys and the
// scores are computed UN-transposed, S = Q_i K_j^T, so a lane holds one key
// column; P and dS, rounded to bf16, are then directly the right-hand operands of
// dV_j^T += dO_i^T P and dK_j^T += Q_i^T dS (contractions over the query rows),
// whose left-hand operands come from transposing LDS reads of the row-major
// Q_i / dO_i tiles. Only dQ_i = dS K_j contracts over keys, i.e. across the
// wavefronts: dS goes through LDS once and every wavefront then forms a
// (32 x 32) tile of dQ_i over all 128 keys.
#include "fa_common.h"
#include "fa_kernels.h"

namespace fa {

__device__ __forceinline__ long stat_index(const Problem& p, long tok, int h) {
  // index of (token, head) in the [B, Hq, N] (dense) or [Hq, T] (ragged) statistics layout
  if (p.cu_seqlens) return (long)h * p.lse_head_stride + tok;
  long b = tok / p.N, r = tok - b * p.N;
  return b * p.lse_seq_stride + (long)h * p.lse_head_stride + r;
}

template <int D>
__global__ __launch_bounds__(256) void bwd_prep_kernel(BwdArgs a) {
  constexpr int LPR = D / 8;  // lanes per row, 8 elements each
  constexpr int RPB = 256 / LPR;
  const long nrows = (long)a.p.total_tokens * a.p.Hq;
  const long row = (long)blockIdx.x * RPB + threadIdx.x / LPR;
  const int c = threadIdx.x % LPR;
  float acc = 0.f;
  if (row < nrows) {
    bf16x8 o = *(const bf16x8*)(a.O + row * D + 8 * c);
    bf16x8 g = *(const bf16x8*)(a.dO + row * D + 8 * c);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc += (float)o[t] * (float)g[t];
    f32x4 z = {0.f, 0.f, 0.f, 0.f};
    *(f32x4*)(a.dQacc + row * D + 8 * c) = z;
    *(f32x4*)(a.dQacc + row * D + 8 * c + 4) = z;
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (row < nrows && c == 0) {
    long tok = row / a.p.Hq;
    int h = (int)(row - tok * a.p.Hq);
    a.Dvec[stat_index(a.p, tok, h)] = acc;
  }
}

template <int D>
__global__ __launch_bounds__(256) void bwd_convert_kernel(BwdArgs a) {
  const long n8 = (long)a.p.total_tokens * a.p.Hq * D / 8;
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  f32x4 x = *(const f32x4*)(a.dQacc + 8 * i);
  f32x4 y = *(const f32x4*)(a.dQacc + 8 * i + 4);
  const float sc = a.p.scale;
  u32x4 r;
  r[0] = pack_bf16(x[0] * sc, x[1] * sc);
  r[1] = pack_bf16(x[2] * sc, x[3] * sc);
  r[2] = pack_bf16(y[0] * sc, y[1] * sc);
  r[3] = pack_bf16(y[2] * sc, y[3] * sc);
  *(u32x4*)(a.dQ + 8 * i) = r;
}

template <int D, int QT, bool CAUSAL>
__global__ __launch_bounds__(256, 1) void bwd_kernel(BwdArgs a) {
  constexpr int BC = 128, BR = 32 * QT;
  constexpr int KS = D / 16, DT = D / 32;
  constexpr int QSTR = D + 8;      // Q_i / dO_i tile pitch (elements)
  constexpr int KSTR = D + 32;     // K_j tile pitch
  constexpr int SSTR = BR + 8;     // dS tile pitch: [key][query]
  constexpr int CPR = D / 8;       // 16-byte chunks per row
  constexpr int NLD = BR * CPR / 256;  // chunks per thread per Q_i (or dO_i) tile
  constexpr int NTILE = DT * QT / 4;   // dQ^T tiles per wavefront
  static_assert(DT * QT % 4 == 0, "dQ tiles must divide over 4 wavefronts");
  static_assert(BR * CPR % 256 == 0, "tile must divide over 256 threads");

  __shared__ __attribute__((aligned(16))) __bf16 Qs[BR * QSTR];
  __shared__ __attribute__((aligned(16))) __bf16 dOs[BR * QSTR];
  __shared__ __attribute__((aligned(16))) __bf16 Ks[BC * KSTR];
  __shared__ __attribute__((aligned(16))) __bf16 dSs[BC * SSTR];
  __shared__ __attribute__((aligned(16))) float Ls[BR];
  __shared__ __attribute__((aligned(16))) float Ds[BR];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int lq = lane & 31, hh = lane >> 5;
  const int g = blockIdx.y, s = blockIdx.z;
  const SeqInfo si = seq_info(p, s);
  const int n = si.n;
  const int j0 = blockIdx.x * BC;
  if (j0 >= n) return;
  const long qstride = (long)p.Hq * D, kstride = (long)p.Hkv * D;
  const __bf16* Kb = a.K + (si.tok0 * p.Hkv + g) * D;
  const __bf16* Vb = a.V + (si.tok0 * p.Hkv + g) * D;

  // ---- K_j, V_j: this wavefront's 32 keys as right-hand operands in registers
  //      (Algorithm 2, line 6), and all of K_j in LDS for the dQ product
  const int key = j0 + 32 * w + lq;  // this lane's key column
  bf16x8 Kf[KS], Vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    if (key < n) {
      Kf[ks] = *(const bf16x8*)(Kb + key * kstride + 16 * ks + 8 * hh);
      Vf[ks] = *(const bf16x8*)(Vb + key * kstride + 16 * ks + 8 * hh);
    } else {
      Kf[ks] = (bf16x8){0};
      Vf[ks] = (bf16x8){0};
    }
  }
  for (int id = tid; id < BC * CPR; id += 256) {
    int r = id / CPR, c = id % CPR;
    u32x4 v = {0, 0, 0, 0};
    if (j0 + r < n) v = *(const u32x4*)(Kb + (long)(j0 + r) * kstride + 8 * c);
    *(u32x4*)(Ks + r * KSTR + 8 * c) = v;
  }

  // ---- dK_j^T, dV_j^T accumulators (line 7): rows = head dim, columns = this wavefront's keys
  f32x16 dKt[DT], dVt[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dKt[dt] = dVt[dt] = (f32x16){0};

  const float c2 = p.scale_log2e;
  const int nrb = (n + BR - 1) / BR;
  const int i_first = CAUSAL ? j0 / BR : 0;  // row blocks entirely above the diagonal are skipped

  for (int hq = g * p.G; hq < (g + 1) * p.G; ++hq) {
    const __bf16* Qb = a.Q + (si.tok0 * p.Hq + hq) * D;
    const __bf16* dOb = a.dO + (si.tok0 * p.Hq + hq) * D;
    const long stat0 = s * p.lse_seq_stride + (long)hq * p.lse_head_stride + (p.cu_seqlens ? si.tok0 : 0);
    float* dQb = a.dQacc + (si.tok0 * p.Hq + hq) * D;

    for (int i = i_first; i < nrb; ++i) {
      const int i0 = i * BR;
      __syncthreads();  // readers of the previous step's tiles are done
      // ---- load Q_i, dO_i, L_i, D_i (line 9)
#pragma unroll
      for (int u = 0; u < NLD; ++u) {
        int id = tid + 256 * u;
        int r = id / CPR, c = id % CPR;
        u32x4 q = {0, 0, 0, 0}, d = {0, 0, 0, 0};
        if (i0 + r < n) {
          q = *(const u32x4*)(Qb + (long)(i0 + r) * qstride + 8 * c);
          d = *(const u32x4*)(dOb + (long)(i0 + r) * qstride + 8 * c);
        }
        *(u32x4*)(Qs + r * QSTR + 8 * c) = q;
        *(u32x4*)(dOs + r * QSTR + 8 * c) = d;
      }
      if (tid < BR) {
        const bool ok = i0 + tid < n;
        // rows past the end get L = +inf so that P = exp2(. - inf) = 0 there
        Ls[tid] = ok ? a.LSE[stat0 + i0 + tid] * kLog2e : INFINITY;
        Ds[tid] = ok ? a.Dvec[stat0 + i0 + tid] : 0.f;
      }
      __syncthreads();

#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        // ---- S = Q_i K_j^T (line 10) and dP = dO_i V_j^T (line 13)
        f32x16 S = {0}, dP = {0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          S = mfma32(lds_frag(Qs, QSTR, 32 * qt, 16 * ks, lane), Kf[ks], S);
          dP = mfma32(lds_frag(dOs, QSTR, 32 * qt, 16 * ks, lane), Vf[ks], dP);
        }
        // ---- P = exp(S - L) (line 11), dS = P o (dP - D) (line 14)
        const bool key_ok = key < n;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int q0 = 32 * qt + 8 * r4 + 4 * hh;
          const f32x4 Lv = *(const f32x4*)(Ls + q0);
          const f32x4 Dv = *(const f32x4*)(Ds + q0);
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int r = 4 * r4 + t;
            float pr = fast_exp2(__builtin_fmaf(S[r], c2, -Lv[t]));
            const bool vis = key_ok && (!CAUSAL || key <= i0 + q0 + t);
            pr = vis ? pr : 0.f;
            S[r] = pr;
            dP[r] = pr * (dP[r] - Dv[t]);
          }
        }
        bf16x8 Pf[2], dSf[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          Pf[s2] = pack8(S, s2);
          dSf[s2] = pack8(dP, s2);
          // dS^T to LDS: row = key, 4 consecutive queries per 8-byte store
          u32x4 v = __builtin_bit_cast(u32x4, dSf[s2]);
          __bf16* dst = dSs + (32 * w + lq) * SSTR + 32 * qt + 4 * hh;
          *(u32x2*)(dst + 8 * (2 * s2)) = (u32x2){v[0], v[1]};
          *(u32x2*)(dst + 8 * (2 * s2 + 1)) = (u32x2){v[2], v[3]};
        }
        // ---- dV_j^T += dO_i^T P (line 12), dK_j^T += Q_i^T dS (line 16)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2) {
            dVt[dt] = mfma32(lds_frag_transposed(dOs, QSTR, 32 * qt + 16 * s2, 32 * dt, lane), Pf[s2], dVt[dt]);
            dKt[dt] = mfma32(lds_frag_transposed(Qs, QSTR, 32 * qt + 16 * s2, 32 * dt, lane), dSf[s2], dKt[dt]);
          }
      }
      __syncthreads();  // dS of all 128 keys is in LDS

      // ---- dQ_i += dS K_j (line 15): each wavefront forms NTILE (32 x 32) tiles over all 128 keys.
      //      Rows = queries, columns = head dim, so one atomic instruction covers two
      //      128-byte row segments of the accumulator.
#pragma unroll
      for (int tt = 0; tt < NTILE; ++tt) {
        const int tile = w + 4 * tt, dt = tile % DT, qt = tile / DT;
        f32x16 acc = {0};
#pragma unroll
        for (int kk = 0; kk < BC / 16; ++kk)
          acc = mfma32(lds_frag_transposed(dSs, SSTR, 16 * kk, 32 * qt, lane),
                       lds_frag_transposed(Ks, KSTR, 16 * kk, 32 * dt, lane), acc);
        float* dst = dQb + 32 * dt + lq;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = i0 + 32 * qt + acc_row(r, hh);
          if (row < n) unsafeAtomicAdd(dst + (long)row * qstride, acc[r]);
        }
      }
    }
  }

  // ---- write dK_j, dV_j (line 18); dK carries the softmax scaling
  if (key < n) {
    __bf16* dKp = a.dK + ((si.tok0 + key) * p.Hkv + g) * D + 4 * hh;
    __bf16* dVp = a.dV + ((si.tok0 + key) * p.Hkv + g) * D + 4 * hh;
    const float sc = p.scale;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 kv, vv;
        kv[0] = pack_bf16(dKt[dt][4 * r4 + 0] * sc, dKt[dt][4 * r4 + 1] * sc);
        kv[1] = pack_bf16(dKt[dt][4 * r4 + 2] * sc, dKt[dt][4 * r4 + 3] * sc);
        vv[0] = pack_bf16(dVt[dt][4 * r4 + 0], dVt[dt][4 * r4 + 1]);
        vv[1] = pack_bf16(dVt[dt][4 * r4 + 2], dVt[dt][4 * r4 + 3]);
        *(u32x2*)(dKp + 32 * dt + 8 * r4) = kv;
        *(u32x2*)(dVp + 32 * dt + 8 * r4) = vv;
      }
  }
}

template <int D, int QT>
static hipError_t launch_bwd_d(const BwdArgs& a, int causal, int stages, hipStream_t st) {
  const long nrows = (long)a.p.total_tokens * a.p.Hq;
  constexpr int RPB = 256 / (D / 8);
  hipError_t e = hipSuccess;
  if (stages & 1) {
    hipLaunchKernelGGL((bwd_prep_kernel<D>), dim3((unsigned)((nrows + RPB - 1) / RPB)), dim3(256), 0, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (stages & 2) {
    dim3 grid((a.p.N + 127) / 128, a.p.Hkv, a.p.nseq);
    if (causal) hipLaunchKernelGGL((bwd_kernel<D, QT, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((bwd_kernel<D, QT, false>), grid, dim3(256), 0, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (stages & 4) {
    const long n8 = nrows * D / 8;
    hipLaunchKernelGGL((bwd_convert_kernel<D>), dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, st, a);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_bwd(const BwdArgs& a, int d, int causal, int stages, hipStream_t st) {
  if (d == 64) return launch_bwd_d<64, 2>(a, causal, stages, st);
  return launch_bwd_d<128, 1>(a, causal, stages, st);
}

}  // namespace fa
