// Head dimension 256 (Algorithms 1 and 2 of the paper, the same arithmetic as fa_fwd.hip and
// fa_bwd.hip): three kernels of their own, because nothing of the d <= 128 kernels' budget
// carries over. A 32-row (or 32-key) slice of a 256-wide accumulator takes 128 registers, the
// operands another 64 to 128, so a wavefront needs the whole register file of its SIMD (512
// registers, one wavefront per SIMD): workgroups of FOUR wavefronts, 128 query rows (forward,
// dQ) or 128 keys (dK/dV) each, and no second wavefront on the SIMD to run the softmax
// while the first one multiplies. The backward loops are plain: wait for the tile, barrier,
// products, P and dS, products, barrier, with the next tile in flight meanwhile (two LDS
// stages); the forward kernel interleaves the exponentials of one block with the MFMAs of its
// neighbours inside its single instruction stream.
//
// A 256-wide tile is kept in LDS as two 128-wide halves side by side (columns 0..127 and
// 128..255 of every row), each in the swizzled layout of fa_lds.h, so the operand addressing
// of the d = 128 kernels applies to each half unchanged.
#include "fa_common.h"
#include "fa_kernels.h"
#include "fa_lds.h"

namespace fa {

namespace {

constexpr int kHalf = 128;          // columns of one half tile
constexpr int kRowB = 2 * kHalf;    // its row bytes
constexpr int kLazyLog2 = 8;        // see FA_FWD_LAZY_LOG2 in fa_fwd.hip

__device__ __forceinline__ float max3f(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// lane constants of the operand addressing inside one half tile (fa_lds.h)
struct LaneAddr {
  int zrow;     // 16-byte row operand: (zrow ^ 32 * ks) + row0 * kRowB
  int zcol[2];  // transposing 8-byte reads: (zcol[u] ^ 64 * dt) + 16 * k4 * kRowB
  __device__ __forceinline__ void init(int lane) {
    const int lq = lane & 31, hh = lane >> 5;
    zrow = lq * kRowB + 16 * (hh ^ swz<kRowB>(lq));
    const int p16 = lane & 15, g16 = (lane >> 4) & 1;
#pragma unroll
    for (int u = 0; u < 2; ++u)
      zcol[u] = swz_off<kRowB>(4 * hh + (p16 >> 2) + 8 * u, 2 * g16 + ((p16 & 3) >> 1)) + 8 * (p16 & 1);
  }
};

}  // namespace

// ---------------------------------------------------------------------------------------------
// Forward (Algorithm 1). Wavefront w owns rows 32 w .. 32 w + 31 of a 128-row block; key blocks
// of 64. LDS: three stages of K_j (left | right half, 16 KiB each) and two of V_j.
template <bool CAUSAL, bool F16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void fwd256_kernel(FwdArgs a) {
  constexpr int D = 256, BR = 128, BC = 64, KS = D / 16, DT = D / 32;
  constexpr int HALFB = BC * kRowB, TILEB = 2 * HALFB;  // one K_j or V_j: left | right
  constexpr int KSTAGES = 3, V_OFF = KSTAGES * TILEB;     // K_j: three stages, V_j: two (160 KiB in all)
  __shared__ __attribute__((aligned(1024))) char smem[V_OFF + 2 * TILEB];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, hh = lane >> 5;
  const int nblk = (p.N + BR - 1) / BR;
  const BlockCoord bc = block_coord<CAUSAL>(nblk, p.Hq, p.nseq, p.G);
  if (!bc.valid) return;
  const int rowblk = nblk - 1 - bc.blk;  // longest causal rows first
  const int h = bc.head, s = bc.seq;
  const SeqInfo si = seq_info(p, s);
  const int n = si.n, nk = si.nk, off = nk - n;
  const int i0 = rowblk * BR;
  if (i0 >= n || nk == 0) return;  // (a sequence without keys: see keyless_rows_kernel)
  const int g = h / p.G;
  const long kstride = (long)p.Hkv * D;
  const __bf16* Kb = a.K + (si.tok0k * p.Hkv + g) * D;
  const __bf16* Vb = a.V + (si.tok0k * p.Hkv + g) * D;

  // Q_i operands in registers (line 4)
  const int prow0 = i0 + 32 * w, row = prow0 + lq;
  const int rowc = row < n ? row : n - 1;  // rows past the end compute on a copy and are never stored
  bf16x8 Qf[KS];
  {
    const __bf16* qp = a.Q + ((si.tok0 + rowc) * p.Hq + h) * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Qf[ks] = *(const bf16x8*)(qp + 16 * ks);
  }
  f32x16 O[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x16){0};
  float m = -INFINITY, l = 0.f;

  const int ncol_all = (nk + BC - 1) / BC;
  int ncol = ncol_all;
  if (CAUSAL) {
    const int last_pos = (i0 + BR < n ? i0 + BR : n) - 1 + off;
    const int c = last_pos / BC + 1;
    ncol = c < ncol_all ? c : ncol_all;
  }
  if (ncol < 1) ncol = 1;  // (more queries than keys is only allowed without the mask)

  TileLoader<kHalf, BC, 4, false> loader;
  loader.init(kstride, w, lane, kHalf / 8);
  // One wavefront per SIMD has to overlap its own matrix and vector work: iteration j issues
  // the MFMAs of O^T += V_{j-1}^T P_{j-1}^T and of S_{j+1}^T while it takes the exponentials of block j
  // (whose maximum it has found just before): one basic block in which the two kinds of
  // instruction alternate in source order, held there by scheduling fences.
  //
  // Copies: iteration j requests V_j (two LDS stages; read in iteration j + 1) and K_{j+3}
  // (three stages; read in iteration j + 2), always the same number of copies, past the end too
  // (rows are clamped, the data is never used), so that the waits can count.
  constexpr int CPT = 2 * TileLoader<kHalf, BC, 4, false>::PER;  // copies per wavefront and tile
  auto issue_k = [&](int j) {
    char* st = smem + (j % KSTAGES) * TILEB;
#pragma unroll
    for (int half = 0; half < 2; ++half) loader.load(st + half * HALFB, Kb + half * kHalf, kstride, j * BC, nk - 1, w, lane);
  };
  auto issue_v = [&](int j) {
    char* st = smem + V_OFF + (j & 1) * TILEB;
#pragma unroll
    for (int half = 0; half < 2; ++half) loader.load(st + half * HALFB, Vb + half * kHalf, kstride, j * BC, nk - 1, w, lane);
  };
  issue_k(0);
  issue_k(1);
  issue_k(2);
  // (iteration 0 multiplies a P of zeros with whatever the V stage of "block -1" holds: zeros)
  for (int o = tid * 16; o < TILEB; o += 256 * 16) *(u32x4*)(smem + V_OFF + TILEB + o) = (u32x4){0, 0, 0, 0};
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) touch(Qf[ks]);

  LaneAddr la;
  la.init(lane);
  const float c2 = p.scale_log2e;
  const int lim_row = CAUSAL ? (row + off < nk - 1 ? row + off : nk - 1) : nk - 1;
  f32x16 Sc[2], Sn[2];   // scores of the current block (turned into P in place) and of the next
  bf16x8 Pp[2][2];       // P of the previous block, rounded: the operand of its O update
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) Pp[kt][0] = Pp[kt][1] = (bf16x8){0};
  auto k_operand = [&](int st, int i) {
    const int ks = i >> 1;
    return lds_b128(smem, ((la.zrow + st + (ks >> 3) * HALFB) ^ (32 * (ks & 7))) + (i & 1) * 32 * kRowB);
  };
  auto v_operand = [&](int vst, int i) {
    const int dt = i >> 2, ro = (16 * (i & 3)) * kRowB;
    const int vb = vst + (dt >> 2) * HALFB;
    return lds_tr_pair(smem, ((la.zcol[0] + vb) ^ (64 * (dt & 3))) + ro, ((la.zcol[1] + vb) ^ (64 * (dt & 3))) + ro);
  };

  wait_vmem_upto<2 * CPT>();
  lds_barrier();  // K_0 has landed
  Sc[0] = Sc[1] = (f32x16){0};
  mfma_stream<2 * KS, 4, 1>([&](int i) { return k_operand(0, i); },
                            [&](int i, bf16x8 x) { Sc[i & 1] = mfma32<F16>(x, Qf[i >> 1], Sc[i & 1]); });
  lds_barrier();  // K_0 has been read by everyone (and the zeros above are in place)

  for (int j = 0; j < ncol; ++j) {
    issue_v(j);
    issue_k(j + 3);  // in flight, oldest first: .. K_{j+1}, V_{j-1} | K_{j+2}, V_j, K_{j+3}
    // ---- the maximum of block j and the reference it is measured against (line 9)
    const int col0 = j * BC;
    if ((CAUSAL && col0 + BC - 1 > prow0 + off) || col0 + BC > nk) {
      const int lim = lim_row - col0 - 4 * hh;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) Sc[kt][r] = 32 * kt + acc_row(r, 0) > lim ? -INFINITY : Sc[kt][r];
    }
    float mx = max3f(Sc[0][0], Sc[0][1], Sc[1][0]);
#pragma unroll
    for (int r = 2; r < 16; r += 2) mx = max3f(mx, Sc[0][r], Sc[0][r + 1]);
    mx = max3f(mx, Sc[1][1], Sc[1][2]);
    mx = fmaxf(mx, Sc[1][3]);
#pragma unroll
    for (int r = 4; r < 16; r += 2) mx = max3f(mx, Sc[1][r], Sc[1][r + 1]);
    mx = max_with_partner32(mx);
    const float m_new = fmaxf(m, mx);
    // (lazy: the reference only moves when some row outgrew it by 2^kLazyLog2; O then is rescaled
    // AFTER this iteration's MFMAs, which still add a block measured against the old reference)
    const bool moved = __builtin_amdgcn_ballot_w64((m_new - m) * c2 > (float)kLazyLog2) != 0;
    float alpha = 1.f;
    if (moved) {
      alpha = fast_exp2((m - m_new) * c2);
      l *= alpha;
      m = m_new;
    }
    const float mc = m * c2;
    wait_vmem_upto<3 * CPT>();
    lds_barrier();  // K_{j+1} and V_{j-1} have landed
    // ---- one basic block: 64 MFMAs (O^T += V_{j-1}^T P_{j-1}^T, line 10; S_{j+1}^T = K_{j+1} Q_i^T, line 8)
    //      with the exponentials of block j between them
    {
      const int vst = V_OFF + ((j + 1) & 1) * TILEB, kst = ((j + 1) % KSTAGES) * TILEB;
      constexpr int NPV = 4 * DT, NS = 2 * KS, AH = 3;
      bf16x8 ring[AH];
      auto operand = [&](int i) { return i < NPV ? v_operand(vst, i) : k_operand(kst, i - NPV); };
#pragma unroll
      for (int i = 0; i < AH; ++i) ring[i] = operand(i);
      __builtin_amdgcn_sched_barrier(0);
      Sn[0] = Sn[1] = (f32x16){0};
      float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
      for (int i = 0; i < NPV + NS; ++i) {
        const bf16x8 cur = ring[i % AH];
        if (i + AH < NPV + NS) ring[i % AH] = operand(i + AH);
        if (i < NPV) {
          O[i >> 2] = mfma32<F16>(cur, Pp[(i >> 1) & 1][i & 1], O[i >> 2]);
        } else {
          const int k = i - NPV;
          Sn[k & 1] = mfma32<F16>(cur, Qf[k >> 1], Sn[k & 1]);
        }
        {  // one exponential of block j behind every second MFMA
          const int e = i / 2, kt = e / 16, r = e % 16;
          if (i & 1) {
            // (the two empty statements tie the exponential to this place: instruction selection
            // would otherwise sink all of them behind the last MFMA, next to their uses)
            float x = Sc[kt][r];
            asm volatile("" : "+v"(x));
            float ex = fast_exp2(__builtin_fmaf(x, c2, -mc));
            asm volatile("" : "+v"(ex));
            Sc[kt][r] = ex;
            if (r & 1) rs1 += ex;
            else rs0 += ex;
          }
        }
        __builtin_amdgcn_sched_barrier(0);  // keep this order: the two kinds of work alternate
      }
      l += rs0 + rs1;
    }
    if (moved) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
    }
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      Pp[kt][0] = pack8<F16>(Sc[kt], 0);
      Pp[kt][1] = pack8<F16>(Sc[kt], 1);
      Sc[kt] = Sn[kt];
    }
    lds_barrier();  // K_{j+1} and V_{j-1} have been read by everyone: their stages may be overwritten
  }

  // ---- the last block's O update
  wait_vmem();
  lds_barrier();
  {
    const int vst = V_OFF + ((ncol - 1) & 1) * TILEB;
    mfma_stream<4 * DT, 3, 2>([&](int i) { return v_operand(vst, i); },
                              [&](int i, bf16x8 x) { O[i >> 2] = mfma32<F16>(x, Pp[(i >> 1) & 1][i & 1], O[i >> 2]); });
  }
  lds_barrier();

  // ---- epilogue (lines 12-15): whole rows through LDS, see store_rows_via_lds
  const float lsum = sum_with_partner32(l);
  const float inv = 1.0f / lsum;
  char* stg = smem + w * (32 * kRowB);
  __bf16* op = a.O + ((si.tok0 + prow0) * p.Hq + h) * D;
#pragma unroll
  for (int half = 0; half < 2; ++half)
    store_rows_via_lds<4, F16>(stg, &O[4 * half], inv, op + half * kHalf, (long)p.Hq * D, n - prow0, kHalf, lane);
  if (row < n && hh == 0)
    a.LSE[s * p.lse_seq_stride + h * p.lse_head_stride + (p.cu_seqlens ? si.tok0 : 0) + row] =
        m * p.scale + fast_log2(lsum) * kLn2;
}

hipError_t launch_fwd256(const FwdArgs& a, int causal, hipStream_t st) {
  dim3 grid(grid_size((a.p.N + 127) / 128, a.p.Hq * a.p.nseq)), block(256);
  if (a.p.f16) {
    if (causal) hipLaunchKernelGGL((fwd256_kernel<true, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((fwd256_kernel<false, true>), grid, block, 0, st, a);
  } else {
    if (causal) hipLaunchKernelGGL((fwd256_kernel<true, false>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((fwd256_kernel<false, false>), grid, block, 0, st, a);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// dQ (Algorithm 2, lines 10-15 for one row block): the forward kernel's skeleton. Wavefront w owns
// rows 32 w .. of a 128-row block with Q_i, dO_i, L_i, D_i in registers; per key block S^T and
// dP^T = V_j dO_i^T, then P and dS, then dQ_i^T += K_j^T dS^T with K_j^T from transposing reads.
template <bool CAUSAL, bool F16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void dq256_kernel(BwdArgs a) {
  constexpr int D = 256, BR = 128, BC = 64, KS = D / 16, DT = D / 32;
  constexpr int HALFB = BC * kRowB, STAGEB = 4 * HALFB;
  __shared__ __attribute__((aligned(1024))) char smem[2 * STAGEB];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, hh = lane >> 5;
  const int nblk = (p.N + BR - 1) / BR;
  const BlockCoord bc = block_coord<CAUSAL>(nblk, p.Hq, p.nseq, p.G);
  if (!bc.valid) return;
  const int rowblk = nblk - 1 - bc.blk;
  const int h = bc.head, s = bc.seq;
  const SeqInfo si = seq_info(p, s);
  const int n = si.n, nk = si.nk, off = nk - n;
  const int i0 = rowblk * BR;
  if (i0 >= n || nk == 0) return;  // (a sequence without keys: see keyless_rows_kernel)
  const int g = h / p.G;
  const long kstride = (long)p.Hkv * D;
  const __bf16* Kb = a.K + (si.tok0k * p.Hkv + g) * D;
  const __bf16* Vb = a.V + (si.tok0k * p.Hkv + g) * D;

  const int prow0 = i0 + 32 * w, row = prow0 + lq;
  const int rowc = row < n ? row : n - 1;
  bf16x8 Qf[KS], dOf[KS];
  {
    const long qo = ((si.tok0 + rowc) * p.Hq + h) * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Qf[ks] = *(const bf16x8*)(a.Q + qo + 16 * ks);
      dOf[ks] = *(const bf16x8*)(a.dO + qo + 16 * ks);
    }
  }
  const long stat = s * p.lse_seq_stride + (long)h * p.lse_head_stride + (p.cu_seqlens ? si.tok0 : 0) + rowc;
  const float Lq = row < n ? a.LSE[stat] * kLog2e : INFINITY;  // rows past the end: P = 0
  const float Dq = a.Dvec[stat];
  f32x16 dQt[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dQt[dt] = (f32x16){0};

  const int ncol_all = (nk + BC - 1) / BC;
  int ncol = ncol_all;
  if (CAUSAL) {
    const int last_pos = (i0 + BR < n ? i0 + BR : n) - 1 + off;
    const int c = last_pos / BC + 1;
    ncol = c < ncol_all ? c : ncol_all;
  }
  if (ncol < 1) ncol = 1;

  TileLoader<kHalf, BC, 4, false> loader;
  loader.init(kstride, w, lane, kHalf / 8);
  constexpr int CPB = 4 * TileLoader<kHalf, BC, 4, false>::PER;
  auto issue_block = [&](int j) {
    char* st = smem + (j & 1) * STAGEB;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      loader.load(st + half * HALFB, Kb + half * kHalf, kstride, j * BC, nk - 1, w, lane);
      loader.load(st + (2 + half) * HALFB, Vb + half * kHalf, kstride, j * BC, nk - 1, w, lane);
    }
  };
  issue_block(0);
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    touch(Qf[ks]);
    touch(dOf[ks]);
  }
  touch(Lq);
  touch(Dq);

  LaneAddr la;
  la.init(lane);
  const float c2 = p.scale_log2e;
  const int wrow_last = prow0 + 31 + off;
  const int lim_row = CAUSAL ? (row + off < nk - 1 ? row + off : nk - 1) : nk - 1;
  f32x16 S[2], dP[2];
  bf16x8 dSf[2][2];

  for (int j = 0; j < ncol; ++j) {
    if (j + 1 < ncol) {
      issue_block(j + 1);
      wait_vmem_upto<CPB>();
    } else {
      wait_vmem();
    }
    lds_barrier();
    if (!CAUSAL || j * BC <= wrow_last) {
      const int st = (j & 1) * STAGEB;
      // ---- S^T = K_j Q_i^T (line 10)
      S[0] = S[1] = dP[0] = dP[1] = (f32x16){0};
      mfma_stream<2 * KS, 4, 1>(
          [&](int i) {
            const int ks = i >> 1;
            return lds_b128(smem, ((la.zrow + st + (ks >> 3) * HALFB) ^ (32 * (ks & 7))) + (i & 1) * 32 * kRowB);
          },
          [&](int i, bf16x8 x) { S[i & 1] = mfma32<F16>(x, Qf[i >> 1], S[i & 1]); });
      // ---- dP^T = V_j dO_i^T (line 13) with P = exp(S - L) (line 11) between its MFMAs (one
      //      instruction stream per SIMD has to overlap its own matrix and vector work)
      {
        constexpr int AH = 4;
        bf16x8 ring[AH];
        auto operand = [&](int i) {
          const int ks = i >> 1;
          return lds_b128(smem, ((la.zrow + st + 2 * HALFB + (ks >> 3) * HALFB) ^ (32 * (ks & 7))) + (i & 1) * 32 * kRowB);
        };
#pragma unroll
        for (int i = 0; i < AH; ++i) ring[i] = operand(i);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2 * KS; ++i) {
          const bf16x8 cur = ring[i % AH];
          if (i + AH < 2 * KS) ring[i % AH] = operand(i + AH);
          dP[i & 1] = mfma32<F16>(cur, dOf[i >> 1], dP[i & 1]);
          float x = S[i >> 4][i & 15];  // (tied in place, see the forward kernel)
          asm volatile("" : "+v"(x));
          float ex = fast_exp2(__builtin_fmaf(x, c2, -Lq));
          asm volatile("" : "+v"(ex));
          S[i >> 4][i & 15] = ex;
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // ---- dS = P o (dP - D) (line 14)
      const int col0 = j * BC;
      const bool need_mask = (CAUSAL && col0 + BC - 1 > prow0 + off) || (col0 + BC > nk);
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        if (need_mask) {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (col0 + 32 * kt + acc_row(r, hh) > lim_row) S[kt][r] = 0.f;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) dP[kt][r] = S[kt][r] * (dP[kt][r] - Dq);
        dSf[kt][0] = pack8<F16>(dP[kt], 0);
        dSf[kt][1] = pack8<F16>(dP[kt], 1);
      }
      // ---- dQ_i^T += K_j^T dS^T (line 15)
      mfma_stream<4 * DT, 3, 2>(
          [&](int i) {
            const int dt = i >> 2, ro = (16 * (i & 3)) * kRowB;
            const int kb = st + (dt >> 2) * HALFB;
            return lds_tr_pair(smem, ((la.zcol[0] + kb) ^ (64 * (dt & 3))) + ro, ((la.zcol[1] + kb) ^ (64 * (dt & 3))) + ro);
          },
          [&](int i, bf16x8 x) { dQt[i >> 2] = mfma32<F16>(x, dSf[(i >> 1) & 1][i & 1], dQt[i >> 2]); });
    }
    lds_barrier();
  }

  char* stg = smem + w * (32 * kRowB);
  __bf16* op = a.dQ + ((si.tok0 + prow0) * p.Hq + h) * D;
#pragma unroll
  for (int half = 0; half < 2; ++half)
    store_rows_via_lds<4, F16>(stg, &dQt[4 * half], p.scale, op + half * kHalf, (long)p.Hq * D, n - prow0, kHalf, lane);
}

// ---------------------------------------------------------------------------------------------
// dK_j, dV_j (Algorithm 2, outer loop over column blocks): a workgroup owns 128 keys of one
// key/value head, wavefront w the 32 keys 32 w .. with their K_j and V_j operands AND the
// dK_j^T, dV_j^T accumulators in registers (384 of them). It walks the query heads of the group
// and, per head, the 32-row tiles Q_i | dO_i (left and right halves, 8 KiB each) that are not
// entirely above the diagonal; L_i and -D_i of the tile's rows sit beside them in LDS.
template <bool CAUSAL, bool F16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void dkdv256_kernel(BwdArgs a) {
  constexpr int D = 256, BC = 128, BR = 32, KS = D / 16, DT = D / 32;
  constexpr int HALFB = BR * kRowB, STAGEB = 4 * HALFB;  // Q left | Q right | dO left | dO right
  constexpr int LS_OFF = 2 * STAGEB, DV_OFF = LS_OFF + 2 * BR * 4, SMEM = DV_OFF + 2 * BR * 4;
  __shared__ __attribute__((aligned(1024))) char smem[SMEM < 4 * 32 * kRowB ? 4 * 32 * kRowB : SMEM];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, hh = lane >> 5;
  const BlockCoord bc = block_coord<CAUSAL>((p.Nk + BC - 1) / BC, p.Hkv, p.nseq);  // causal: block 0 is the longest
  if (!bc.valid) return;
  const int g = bc.head, s = bc.seq;
  const SeqInfo si = seq_info(p, s);
  const int n = si.n, nk = si.nk, off = nk - n;
  const int j0 = bc.blk * BC;
  if (j0 >= nk) return;
  const long qstride = (long)p.Hq * D;
  const float c2 = p.scale_log2e;
  const int nrt = (n + BR - 1) / BR;
  int i_first = CAUSAL && j0 > off ? (j0 - off) / BR : 0;  // row tiles entirely above the diagonal are skipped
  if (i_first > nrt) i_first = nrt;
  const int per_head = nrt - i_first, T = per_head * p.G;
  const long stat_base = s * p.lse_seq_stride + (p.cu_seqlens ? si.tok0 : 0);

  // K_j, V_j operands of this lane's key (line 6): registers for the whole kernel
  const int key0 = j0 + 32 * w, key = key0 + lq;
  const bool key_ok = key < nk;
  bf16x8 Kf[KS], Vf[KS];
  {
    const long ko = ((si.tok0k + (key_ok ? key : nk - 1)) * p.Hkv + g) * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Kf[ks] = *(const bf16x8*)(a.K + ko + 16 * ks);
      Vf[ks] = *(const bf16x8*)(a.V + ko + 16 * ks);
    }
  }
  f32x16 dKt[DT], dVt[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dKt[dt] = dVt[dt] = (f32x16){0};

  // tile t = (head g G + t / per_head, row tile i_first + t % per_head)
  float lraw = 0.f, draw = 0.f;
  bool stat_ok = false;
  // (tiles are requested in order: the head and row tile of the next request are carried along, and
  // the per-lane offsets of an interior tile are computed once, so that a request costs a scalar base
  // address and the copy instructions; only the last row tile of a sequence clamps its rows)
  TileLoader<kHalf, BR, 4, false> qloader;
  qloader.init(qstride, w, lane, kHalf / 8);
  int next_hq = g * p.G, next_it = i_first;
  auto issue_tile = [&](int t) {
    const int hq = next_hq, it = next_it;
    if (++next_it == nrt) {
      next_it = i_first;
      ++next_hq;
    }
    char* st = smem + (t & 1) * STAGEB;
    const long head0 = (si.tok0 * p.Hq + hq) * D;  // row 0 of this head
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      qloader.load(st + half * HALFB, a.Q + head0 + half * kHalf, qstride, it * BR, n - 1, w, lane);
      qloader.load(st + (2 + half) * HALFB, a.dO + head0 + half * kHalf, qstride, it * BR, n - 1, w, lane);
    }
    if (tid < BR) {
      const int r = it * BR + tid;
      stat_ok = r < n;
      const long si_ = stat_base + (long)hq * p.lse_head_stride + (stat_ok ? r : n - 1);
      lraw = a.LSE[si_];
      draw = a.Dvec[si_];
    }
  };
  if (T > 0) issue_tile(0);
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    touch(Kf[ks]);
    touch(Vf[ks]);
  }

  LaneAddr la;
  la.init(lane);
  f32x16 S, dP;
  bf16x8 Pf[2], dSf[2];

  int cur_it = i_first;  // row tile of tile t
  for (int t = 0; t < T; ++t) {
    wait_vmem();  // tile t and its statistics have arrived
    touch(lraw);
    touch(draw);
    if (tid < BR) {
      // L in the exponent's base; rows past the end get L = +inf so that P = 0. D is stored
      // negated: it is the initial value of the dP accumulator (line 14).
      *(float*)(smem + LS_OFF + ((t & 1) * BR + tid) * 4) = stat_ok ? lraw * kLog2e : INFINITY;
      *(float*)(smem + DV_OFF + ((t & 1) * BR + tid) * 4) = stat_ok ? -draw : 0.f;
    }
    lds_barrier();
    if (t + 1 < T) issue_tile(t + 1);  // into the other stage, which everyone left at the last barrier
    const int st = (t & 1) * STAGEB;
    const int r0 = cur_it * BR;  // first query row of the tile
    if (++cur_it == nrt) cur_it = i_first;
    // ---- S = Q_i K_j^T (line 10)
    S = (f32x16){0};
    mfma_stream<KS, 4, 1>(
        [&](int i) { return lds_b128(smem, (la.zrow + st + (i >> 3) * HALFB) ^ (32 * (i & 7))); },
        [&](int i, bf16x8 x) { S = mfma32<F16>(x, Kf[i], S); });
    // ---- dP - D = dO_i V_j^T - D (lines 13, 14; -D is where the accumulator starts) with
    //      P = exp(S - L) (line 11) between its MFMAs: one instruction stream per SIMD has to
    //      overlap its own matrix and vector work (see the forward kernel)
    f32x4 Lv[4];
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const f32x4 Dn = *(const f32x4*)(smem + DV_OFF + ((t & 1) * BR + 8 * r4 + 4 * hh) * 4);
      Lv[r4] = *(const f32x4*)(smem + LS_OFF + ((t & 1) * BR + 8 * r4 + 4 * hh) * 4);
#pragma unroll
      for (int u = 0; u < 4; ++u) dP[4 * r4 + u] = Dn[u];
    }
    {
      constexpr int AH = 4;
      bf16x8 ring[AH];
      auto operand = [&](int i) { return lds_b128(smem, (la.zrow + st + 2 * HALFB + (i >> 3) * HALFB) ^ (32 * (i & 7))); };
#pragma unroll
      for (int i = 0; i < AH; ++i) ring[i] = operand(i);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        const bf16x8 cur = ring[i % AH];
        if (i + AH < KS) ring[i % AH] = operand(i + AH);
        dP = mfma32<F16>(cur, Vf[i], dP);
        float x = S[i];  // (tied in place, see the forward kernel)
        asm volatile("" : "+v"(x));
        float ex = fast_exp2(__builtin_fmaf(x, c2, -Lv[i >> 2][i & 3]));
        asm volatile("" : "+v"(ex));
        S[i] = ex;
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if ((CAUSAL && key0 + 31 > r0 + off) || j0 + BC > nk) {
      // visible: key < nk and (causal) key <= r0 + off + row of the tile, row = acc_row(r, hh)
      const int kc = key_ok ? (CAUSAL ? key - (r0 + off) - 4 * hh : -1) : 0x7fffffff;
#pragma unroll
      for (int r = 0; r < 16; ++r) S[r] = kc <= acc_row(r, 0) ? S[r] : 0.f;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) dP[r] *= S[r];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      Pf[s2] = pack8<F16>(S, s2);
      dSf[s2] = pack8<F16>(dP, s2);
    }
    // ---- dV_j^T += dO_i^T P (line 12), dK_j^T += Q_i^T dS (line 16)
    mfma_stream<4 * DT, 3, 2>(
        [&](int i) {
          const int k = i >> 1, dt = k >> 1, s2 = k & 1;
          const int qoff = st + ((i & 1) ? 2 : 0) * HALFB + (dt >> 2) * HALFB + 16 * s2 * kRowB;
          return lds_tr_pair(smem, (la.zcol[0] + qoff) ^ (64 * (dt & 3)), (la.zcol[1] + qoff) ^ (64 * (dt & 3)));
        },
        [&](int i, bf16x8 x) {
          const int k = i >> 1, dt = k >> 1, s2 = k & 1;
          if (i & 1) dVt[dt] = mfma32<F16>(x, Pf[s2], dVt[dt]);
          else dKt[dt] = mfma32<F16>(x, dSf[s2], dKt[dt]);
        });
    lds_barrier();  // the tile has been read by everyone
  }

  // ---- write dK_j, dV_j (line 18); dK carries the scaling
  wait_vmem();
  lds_barrier();
  char* stg = smem + w * (32 * kRowB);
  const long kvoff = ((si.tok0k + key0) * p.Hkv + g) * D;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    store_rows_via_lds<4, F16>(stg, &dKt[4 * half], p.scale, a.dK + kvoff + half * kHalf, (long)p.Hkv * D, nk - key0, kHalf, lane);
    store_rows_via_lds<4, F16>(stg, &dVt[4 * half], 1.f, a.dV + kvoff + half * kHalf, (long)p.Hkv * D, nk - key0, kHalf, lane);
  }
}

hipError_t launch_bwd256(const BwdArgs& a, int causal, int stages, hipStream_t st) {
  hipError_t e = hipSuccess;
  if (stages & 2) {
    dim3 grid(grid_size((a.p.Nk + 127) / 128, a.p.Hkv * a.p.nseq)), block(256);
    if (a.p.f16) {
      if (causal) hipLaunchKernelGGL((dkdv256_kernel<true, true>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((dkdv256_kernel<false, true>), grid, block, 0, st, a);
    } else {
      if (causal) hipLaunchKernelGGL((dkdv256_kernel<true, false>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((dkdv256_kernel<false, false>), grid, block, 0, st, a);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (stages & 4) {
    dim3 grid(grid_size((a.p.N + 127) / 128, a.p.Hq * a.p.nseq)), block(256);
    if (a.p.f16) {
      if (causal) hipLaunchKernelGGL((dq256_kernel<true, true>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((dq256_kernel<false, true>), grid, block, 0, st, a);
    } else {
      if (causal) hipLaunchKernelGGL((dq256_kernel<true, false>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((dq256_kernel<false, false>), grid, block, 0, st, a);
    }
    e = hipGetLastError();
  }
  return e;
}

}  // namespace fa
