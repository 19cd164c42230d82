// Forward pass of exact attention for gfx950 (Algorithm 1 of the paper).
//
// One workgroup (4 wavefronts) owns one block of BR = 128 * NQ query rows of one
// (sequence, query head) and walks the key/value sequence in blocks of BC = 64
// (the inner loop over column blocks j; the outer loop over row blocks i is the
// grid, section 3.2 "Forward pass"). Each wavefront owns 32 * NQ whole query
// rows, so no reduction between wavefronts is ever needed (section 3.3).
//
// The scores are computed TRANSPOSED, S^T = K_j Q_i^T, with 32x32x16 bf16 MFMAs:
// a lane then holds 16 keys of ONE query per 32x32 tile, the row maximum and row
// sum are in-lane reductions plus a single exchange with lane ^ 32, and the
// exponentiated tile, rounded to bf16, is already in the operand layout of the
// second product O^T += V_j^T P^T. V_j^T operands come from transposing LDS reads
// of the row-major V tile, so nothing is ever transposed in memory.
#include "fa_common.h"
#include "fa_kernels.h"

namespace fa {

template <int D, int NQ, bool CAUSAL>
__global__ __launch_bounds__(256, (NQ == 1 ? 2 : 1)) void fwd_kernel(FwdArgs a) {
  constexpr int BR = 128 * NQ, BC = 64;
  constexpr int KSTR = D + 8;    // K tile row pitch (elements): 16 B pad, conflict-free b128 row reads
  constexpr int VSTR = D + 32;   // V tile row pitch: 64 B pad, conflict-free transposing reads
  constexpr int KS = D / 16;     // contraction steps of the first product
  constexpr int DT = D / 32;     // 32-row tiles of O^T
  constexpr int CPR = D / 8;     // 16-byte chunks per tile row
  constexpr int NLD = BC * CPR / 256;  // chunks each thread stages per tile

  __shared__ __attribute__((aligned(16))) __bf16 Ks[BC * KSTR];
  __shared__ __attribute__((aligned(16))) __bf16 Vs[BC * VSTR];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int lq = lane & 31, hh = lane >> 5;
  const int nblk = (p.N + BR - 1) / BR;
  const BlockCoord bc = block_coord<CAUSAL>(nblk, p.Hq);
  const int rowblk = nblk - 1 - bc.blk;  // longest causal rows first
  const int h = bc.head, s = bc.seq;
  const SeqInfo si = seq_info(p, s);
  const int n = si.n;
  const int i0 = rowblk * BR;
  if (i0 >= n) return;
  const int g = h / p.G;
  const long qstride = (long)p.Hq * D, kstride = (long)p.Hkv * D;
  const __bf16* Qb = a.Q + (si.tok0 * p.Hq + h) * D;
  const __bf16* Kb = a.K + (si.tok0 * p.Hkv + g) * D;
  const __bf16* Vb = a.V + (si.tok0 * p.Hkv + g) * D;

  // ---- Q_i fragments: registers for the whole kernel (Algorithm 1, line 4)
  bf16x8 Qf[NQ][KS];
  const int wrow0 = i0 + w * 32 * NQ;  // first query row of this wavefront
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    int row = wrow0 + 32 * qt + lq;
    row = row < n ? row : n - 1;  // rows past the end compute on a copy and are never stored
    const __bf16* qp = Qb + row * qstride + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Qf[qt][ks] = *(const bf16x8*)(qp + 16 * ks);
  }

  // ---- on-chip state (Algorithm 1, line 5)
  f32x16 O[NQ][DT];
  float m[NQ], l[NQ];  // running row maximum (raw score units) and this lane's share of the row sum
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    m[qt] = -INFINITY;
    l[qt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[qt][dt] = (f32x16){0};
  }

  // column blocks to visit: all of them, or (causal) those not entirely above the diagonal
  const int ncol_all = (n + BC - 1) / BC;
  int ncol = ncol_all;
  if (CAUSAL) {
    int last_row = (i0 + BR < n ? i0 + BR : n) - 1;
    int c = last_row / BC + 1;
    ncol = c < ncol_all ? c : ncol_all;
  }

  // ---- staging: each thread moves NLD 16-byte chunks of K and of V per tile
  u32x4 kreg[NLD], vreg[NLD];
  auto load_tile = [&](int j) {
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
      int id = tid + 256 * u;
      int r = id / CPR, c = id % CPR;
      int key = j * BC + r;
      if (key < n) {
        kreg[u] = *(const u32x4*)(Kb + key * kstride + 8 * c);
        vreg[u] = *(const u32x4*)(Vb + key * kstride + 8 * c);
      } else {
        kreg[u] = (u32x4){0, 0, 0, 0};
        vreg[u] = (u32x4){0, 0, 0, 0};
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
      int id = tid + 256 * u;
      int r = id / CPR, c = id % CPR;
      *(u32x4*)(Ks + r * KSTR + 8 * c) = kreg[u];
      *(u32x4*)(Vs + r * VSTR + 8 * c) = vreg[u];
    }
  };

  load_tile(0);
  store_tile();
  __syncthreads();

  const float c2 = p.scale_log2e;
  const int wrow_last = wrow0 + 32 * NQ - 1;

  for (int j = 0; j < ncol; ++j) {
    if (j + 1 < ncol) load_tile(j + 1);  // in flight while this tile is computed

    const int col0 = j * BC;
    const bool active = !CAUSAL || col0 <= wrow_last;  // else every score of this wavefront is masked
    if (active) {
      // ---- S^T = K_j Q_i^T (Algorithm 1, line 8)
      f32x16 S[NQ][2];
#pragma unroll
      for (int qt = 0; qt < NQ; ++qt) S[qt][0] = S[qt][1] = (f32x16){0};
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          bf16x8 kf = lds_frag(Ks, KSTR, 32 * kt, 16 * ks, lane);
#pragma unroll
          for (int qt = 0; qt < NQ; ++qt) S[qt][kt] = mfma32(kf, Qf[qt][ks], S[qt][kt]);
        }

      // ---- mask: causal entries above the diagonal and columns past the end
      const bool need_mask = (CAUSAL && col0 + BC - 1 > wrow0) || (col0 + BC > n);
      if (need_mask) {
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
          const int row = wrow0 + 32 * qt + lq;
          const int lim = CAUSAL ? (row < n - 1 ? row : n - 1) : n - 1;  // last visible column
#pragma unroll
          for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              int col = col0 + 32 * kt + acc_row(r, hh);
              if (col > lim) S[qt][kt][r] = -INFINITY;
            }
        }
      }

      // ---- online softmax (Algorithm 1, line 9) and rescale of O (line 10)
      bf16x8 Pf[NQ][2][2];
#pragma unroll
      for (int qt = 0; qt < NQ; ++qt) {
        float mx = S[qt][0][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S[qt][0][r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[qt][1][r]);
        mx = max_with_partner32(mx);
        const float m_new = fmaxf(m[qt], mx);
        // column 0 is visible to every row and tiles are walked in ascending order,
        // so m_new is finite from the first tile on and exp2(-inf) = 0 covers the start.
        if (__builtin_amdgcn_ballot_w64(m_new != m[qt]) != 0) {
          const float alpha = fast_exp2((m[qt] - m_new) * c2);
          l[qt] *= alpha;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[qt][dt][r] *= alpha;
          m[qt] = m_new;
        }
        const float mc = m_new * c2;
        float rs = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float e = fast_exp2(__builtin_fmaf(S[qt][kt][r], c2, -mc));
            S[qt][kt][r] = e;
            rs += e;
          }
          Pf[qt][kt][0] = pack8(S[qt][kt], 0);
          Pf[qt][kt][1] = pack8(S[qt][kt], 1);
        }
        l[qt] += rs;
      }

      // ---- O^T += V_j^T P^T (Algorithm 1, line 10)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2) {
            bf16x8 vf = lds_frag_transposed(Vs, VSTR, 32 * kt + 16 * s2, 32 * dt, lane);
#pragma unroll
            for (int qt = 0; qt < NQ; ++qt) O[qt][dt] = mfma32(vf, Pf[qt][kt][s2], O[qt][dt]);
          }
    }

    __syncthreads();  // everyone is done reading tile j
    if (j + 1 < ncol) store_tile();
    __syncthreads();
  }

  // ---- epilogue: O = diag(l)^-1 O, L = m + log l (Algorithm 1, lines 12-15)
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    const int row = wrow0 + 32 * qt + lq;
    const float lsum = sum_with_partner32(l[qt]);
    const float inv = 1.0f / lsum;
    if (row < n) {
      __bf16* op = a.O + ((si.tok0 + row) * p.Hq + h) * D;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 v;
          v[0] = pack_bf16(O[qt][dt][4 * q4 + 0] * inv, O[qt][dt][4 * q4 + 1] * inv);
          v[1] = pack_bf16(O[qt][dt][4 * q4 + 2] * inv, O[qt][dt][4 * q4 + 3] * inv);
          *(u32x2*)(op + 32 * dt + 8 * q4 + 4 * hh) = v;
        }
      if (hh == 0)
        a.LSE[s * p.lse_seq_stride + h * p.lse_head_stride + (p.cu_seqlens ? si.tok0 : 0) + row] =
            m[qt] * p.scale + fast_log2(lsum) * kLn2;
    }
  }
}

template <int D, int NQ>
static hipError_t launch_fwd_nq(const FwdArgs& a, int causal, hipStream_t st) {
  constexpr int BR = 128 * NQ;
  dim3 grid((unsigned)((a.p.N + BR - 1) / BR) * a.p.Hq * a.p.nseq), block(256);
  if (causal) hipLaunchKernelGGL((fwd_kernel<D, NQ, true>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((fwd_kernel<D, NQ, false>), grid, block, 0, st, a);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdArgs& a, int d, int causal, hipStream_t st) {
  const int nq = a.cfg_nq;
  if (d == 64) return nq == 2 ? launch_fwd_nq<64, 2>(a, causal, st) : launch_fwd_nq<64, 1>(a, causal, st);
  return nq == 2 ? launch_fwd_nq<128, 2>(a, causal, st) : launch_fwd_nq<128, 1>(a, causal, st);
}

}  // namespace fa
