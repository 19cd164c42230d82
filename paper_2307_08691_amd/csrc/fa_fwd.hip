// Forward pass of exact attention for gfx950 (Algorithm 1 of the paper).
//
// One workgroup (4 wavefronts) owns one block of BR = 128 query rows of one
// (sequence, query head) and walks the key/value sequence in blocks of BC = 64
// (the inner loop over column blocks j; the outer loop over row blocks i is the
// grid, section 3.2 "Forward pass"). Each wavefront owns 32 whole query rows, so
// no reduction between wavefronts is ever needed (section 3.3). Two workgroups
// share a CU: while one wavefront of a SIMD runs MFMAs the other does softmax.
//
// The scores are computed TRANSPOSED, S^T = K_j Q_i^T, with 32x32x16 bf16 MFMAs:
// a lane then holds 16 keys of ONE query per 32x32 tile, the row maximum and row
// sum are in-lane reductions plus a single exchange with lane ^ 32, and the
// exponentiated tile, rounded to bf16, is already in the operand layout of the
// second product O^T += V_j^T P^T. V_j^T operands come from transposing LDS reads
// of the row-major V tile, so nothing is ever transposed in memory.
//
// K_j and V_j travel HBM -> LDS directly (no registers), one tile ahead, into the
// other half of a double buffer; the tiles are swizzled, not padded.
#include "fa_common.h"
#include "fa_kernels.h"
#include "fa_lds.h"

namespace fa {

__device__ __forceinline__ float max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void fwd_kernel(FwdArgs a) {
  constexpr int BR = 128, BC = 64;
  constexpr int KS = D / 16;  // contraction steps of the first product
  constexpr int DT = D / 32;  // 32-row tiles of O^T
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = BC * ROWB, BUFB = 2 * TILEB;  // one buffer = K_j | V_j

  __shared__ __attribute__((aligned(1024))) char smem[2 * BUFB];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
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
  const long kstride = (long)p.Hkv * D;
  const __bf16* Kb = a.K + (si.tok0 * p.Hkv + g) * D;
  const __bf16* Vb = a.V + (si.tok0 * p.Hkv + g) * D;

  // ---- Q_i operands: registers for the whole kernel (Algorithm 1, line 4)
  const int wrow0 = i0 + 32 * w;  // first query row of this wavefront
  const int row = wrow0 + lq;
  const int rowc = row < n ? row : n - 1;  // rows past the end compute on a copy and are never stored
  bf16x8 Qf[KS];
  {
    const __bf16* qp = a.Q + ((si.tok0 + rowc) * p.Hq + h) * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Qf[ks] = *(const bf16x8*)(qp + 16 * ks);
  }

  // ---- on-chip state (Algorithm 1, line 5)
  f32x16 O[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x16){0};
  float m = -INFINITY;  // running row maximum, raw score units
  float l = 0.f;        // this lane's share of the row sum (the two lane halves are added at the end)

  // column blocks to visit: all of them, or (causal) those not entirely above the diagonal
  const int ncol_all = (n + BC - 1) / BC;
  int ncol = ncol_all;
  if (CAUSAL) {
    const int last_row = (i0 + BR < n ? i0 + BR : n) - 1;
    const int c = last_row / BC + 1;
    ncol = c < ncol_all ? c : ncol_all;
  }

  auto issue_loads = [&](int j, int buf) {
    tile_load_async<D, BC, 4>(smem + buf * BUFB, Kb, kstride, j * BC, n - 1, w, lane);
    tile_load_async<D, BC, 4>(smem + buf * BUFB + TILEB, Vb, kstride, j * BC, n - 1, w, lane);
  };
  issue_loads(0, 0);
  wait_vmem();
  lds_barrier();

  // lane constants of the LDS addressing (see fa_lds.h)
  const int zrow = lq * ROWB + 16 * (hh ^ swz<ROWB>(lq));
  const int p16 = lane & 15, g16 = (lane >> 4) & 1;
  int zcol[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
    zcol[u] = swz_off<ROWB>(4 * hh + (p16 >> 2) + 8 * u, 2 * g16 + ((p16 & 3) >> 1)) + 8 * (p16 & 1);

  const float c2 = p.scale_log2e;
  const int wrow_last = wrow0 + 31;
  const int lim_row = CAUSAL ? (row < n - 1 ? row : n - 1) : n - 1;  // last visible column of this lane's row

  for (int j = 0; j < ncol; ++j) {
    const int buf = j & 1;
    if (j + 1 < ncol) issue_loads(j + 1, buf ^ 1);  // in flight while this tile is computed
    const int col0 = j * BC;
    const bool active = !CAUSAL || col0 <= wrow_last;  // else every score of this wavefront is masked
    if (active) {
      const int zk = zrow + buf * BUFB;
      const int zv0 = zcol[0] + buf * BUFB + TILEB, zv1 = zcol[1] + buf * BUFB + TILEB;

      // ---- S^T = K_j Q_i^T (Algorithm 1, line 8)
      f32x16 S[2];
      S[0] = S[1] = (f32x16){0};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        S[0] = mfma32(lds_b128(smem, zk ^ (32 * ks)), Qf[ks], S[0]);
        S[1] = mfma32(lds_b128(smem, (zk ^ (32 * ks)) + 32 * ROWB), Qf[ks], S[1]);
      }

      // ---- mask: causal entries above the diagonal and columns past the end
      const bool need_mask = (CAUSAL && col0 + BC - 1 > wrow0) || (col0 + BC > n);
      if (need_mask) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (col0 + 32 * kt + acc_row(r, hh) > lim_row) S[kt][r] = -INFINITY;
      }

      // ---- online softmax (Algorithm 1, line 9) and rescale of O (line 10)
      float mx = max3(S[0][0], S[0][1], S[1][0]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = max3(mx, S[0][r], S[0][r + 1]);
      mx = max3(mx, S[1][1], S[1][2]);
      mx = fmaxf(mx, S[1][3]);
#pragma unroll
      for (int r = 4; r < 16; r += 2) mx = max3(mx, S[1][r], S[1][r + 1]);
      mx = max_with_partner32(mx);
      const float m_new = fmaxf(m, mx);
      // column 0 is visible to every row and tiles are walked in ascending order,
      // so m_new is finite from the first tile on and exp2(-inf) = 0 covers the start.
      if (__builtin_amdgcn_ballot_w64(m_new != m) != 0) {
        const float alpha = fast_exp2((m - m_new) * c2);
        l *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
        m = m_new;
      }
      const float mc = m_new * c2;
      bf16x8 Pf[2][2];
      float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float e0 = fast_exp2(__builtin_fmaf(S[kt][r], c2, -mc));
          const float e1 = fast_exp2(__builtin_fmaf(S[kt][r + 1], c2, -mc));
          S[kt][r] = e0;
          S[kt][r + 1] = e1;
          rs0 += e0;
          rs1 += e1;
        }
        Pf[kt][0] = pack8(S[kt], 0);
        Pf[kt][1] = pack8(S[kt], 1);
      }
      l += rs0 + rs1;

      // ---- O^T += V_j^T P^T (Algorithm 1, line 10)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2) {
            const int ro = (32 * kt + 16 * s2) * ROWB;
            O[dt] = mfma32(lds_tr_pair(smem, (zv0 ^ (64 * dt)) + ro, (zv1 ^ (64 * dt)) + ro), Pf[kt][s2], O[dt]);
          }
    }
    wait_vmem();
    lds_barrier();  // next tiles visible; this step's tiles are free
  }

  // ---- epilogue: O = diag(l)^-1 O, L = m + log l (Algorithm 1, lines 12-15)
  const float lsum = sum_with_partner32(l);
  const float inv = 1.0f / lsum;
  if (row < n) {
    __bf16* op = a.O + ((si.tok0 + row) * p.Hq + h) * D + 4 * hh;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 o;
        o[0] = pack_bf16(O[dt][4 * r4 + 0] * inv, O[dt][4 * r4 + 1] * inv);
        o[1] = pack_bf16(O[dt][4 * r4 + 2] * inv, O[dt][4 * r4 + 3] * inv);
        *(u32x2*)(op + 32 * dt + 8 * r4) = o;
      }
    if (hh == 0)
      a.LSE[s * p.lse_seq_stride + h * p.lse_head_stride + (p.cu_seqlens ? si.tok0 : 0) + row] =
          m * p.scale + fast_log2(lsum) * kLn2;
  }
}

template <int D>
static hipError_t launch_fwd_d(const FwdArgs& a, int causal, hipStream_t st) {
  dim3 grid((unsigned)((a.p.N + 127) / 128) * a.p.Hq * a.p.nseq), block(256);
  if (causal) hipLaunchKernelGGL((fwd_kernel<D, true>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((fwd_kernel<D, false>), grid, block, 0, st, a);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdArgs& a, int d, int causal, hipStream_t st) {
  return d == 64 ? launch_fwd_d<64>(a, causal, st) : launch_fwd_d<128>(a, causal, st);
}

}  // namespace fa
