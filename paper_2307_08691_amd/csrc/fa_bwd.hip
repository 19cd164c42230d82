// Backward pass of exact attention for gfx950 (Algorithm 2 of the paper).
//
// Three launches on the caller's stream:
//   1. prep:  D = rowsum(dO o O) (Algorithm 2, line 4)
//   2. dK/dV: one workgroup per block of 128 keys of one (sequence, key/value head)
//             (section 3.2 "Backward pass"); it loops over the query heads that share the
//             key/value head and over the row blocks i, recomputes P from the saved
//             logsumexp (line 11) and keeps dK_j, dV_j in MFMA accumulators for the whole
//             loop (lines 12-16 without line 15)
//   3. dQ:    one workgroup per block of 128 query rows; it loops over the column blocks,
//             recomputes P and dS and keeps dQ_i in MFMA accumulators (line 15)
//
// The paper accumulates dQ from the column-block workers with atomic adds (section 3.2).
// On MI355X float32 atomics into L2 retire at roughly 1.3 TB/s chip-wide: with them the
// single-kernel form of Algorithm 2 spent more than half its time waiting for the atomic
// unit (6.8 ms against 3.1 ms with the atomics removed, d = 128, N = 8192, 32 heads). The
// dQ pass here instead recomputes S and dP (7 products instead of 5) and needs no
// cross-workgroup accumulation at all; dQ, dK and dV are bit-reproducible.
//
// Lane layouts. dK/dV kernel: scores are computed UN-transposed, S = Q_i K_j^T, so a lane
// holds one key column; P and dS, rounded to bf16, are directly the right-hand operands of
// dV_j^T += dO_i^T P and dK_j^T += Q_i^T dS (contractions over the query rows), whose
// left-hand operands come from transposing LDS reads of the row-major Q_i / dO_i tiles.
// dQ kernel: scores are computed transposed, S^T = K_j Q_i^T, so a lane holds one query
// row (L_i, D_i are per-lane scalars) and dS^T in bf16 is the right-hand operand of
// dQ_i^T += K_j^T dS^T, with K_j^T from transposing reads of the K tile.
#include "fa_common.h"
#include "fa_kernels.h"
#include "fa_lds.h"

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
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (row < nrows && c == 0) {
    long tok = row / a.p.Hq;
    int h = (int)(row - tok * a.p.Hq);
    a.Dvec[stat_index(a.p, tok, h)] = acc;
  }
}


// dK/dV kernel: 8 wavefronts, two per SIMD so that one can run MFMAs while the other
// does the elementwise work. Wavefront (kg, qh) owns keys 32*kg.. of the column block
// and the query tiles qh*QTW.. of each step.
//
// LDS addressing. Every tile is swizzled (see swz<>). Because the XOR only touches
// address bits 4..7 while row offsets live in bits >= 7/8, the address of every MFMA
// operand is (lane constant) ^ (compile-time constant) + (immediate): the lane
// constants are a handful of registers computed once, instead of one register per
// distinct operand.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(512) void bwd_dkdv_kernel(BwdArgs a) {
  constexpr int BC = 128;               // keys per workgroup
  constexpr int QTW = D == 128 ? 1 : 2;  // 32-row query tiles per wavefront per step
  constexpr int BR = 64 * QTW;          // query rows per step
  constexpr int KS = D / 16, DT = D / 32;
  constexpr int ROWB = 2 * D;           // row bytes of the Q_i, dO_i, K_j, V_j tiles
  // byte offsets inside the LDS block
  constexpr int KT_OFF = 0, VT_OFF = BC * ROWB, QDO_OFF = 2 * BC * ROWB;
  constexpr int TILEB = BR * ROWB, BUFB = 2 * TILEB;  // one Q_i (or dO_i) tile; one buffer = Q_i | dO_i
  constexpr int LS_OFF = QDO_OFF + 2 * BUFB, DV_OFF = LS_OFF + 2 * BR * 4;
  constexpr int SMEM = DV_OFF + 2 * BR * 4;
  static_assert(VT_OFF + BC * ROWB <= 65536 && BUFB <= 32768, "immediate offsets must fit 16 bits");

  __shared__ __attribute__((aligned(1024))) char smem[SMEM];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int v = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = v & 3, qh = v >> 2;
  const int lq = lane & 31, hh = lane >> 5;
  const BlockCoord bc = block_coord<CAUSAL>((p.N + BC - 1) / BC, p.Hkv, p.nseq);  // causal: block 0 is the longest
  if (!bc.valid) return;
  const int g = bc.head, s = bc.seq;
  const SeqInfo si = seq_info(p, s);
  const int n = si.n;
  const int j0 = bc.blk * BC;
  if (j0 >= n) return;
  const long qstride = (long)p.Hq * D, kstride = (long)p.Hkv * D;

  const float c2 = p.scale_log2e;
  const int nrb = (n + BR - 1) / BR;
  const int i_first = CAUSAL ? j0 / BR : 0;  // row blocks entirely above the diagonal are skipped
  const int per_head = nrb - i_first;
  const int nsteps = per_head * p.G;
  const long stat_base = s * p.lse_seq_stride + (p.cu_seqlens ? si.tok0 : 0);

  // Q_i, dO_i (line 9) go HBM -> LDS directly, one step ahead, into the other buffer;
  // L_i, D_i travel through two registers of the first BR threads.
  // The raw statistics are only touched (scaled, masked) when they are committed to LDS at
  // the end of the step: using them earlier would make the compiler wait for them right
  // after the tile copies were issued, i.e. for the copies themselves.
  float lraw = 0.f, draw = 0.f;
  bool stat_ok = false;
  TileLoader<D, BR, 8> qloader;  // Q_i and dO_i tiles have the same shape and row pitch
  qloader.init(qstride, v, lane);
  auto issue_loads = [&](int t, int buf) {
    const int hq = g * p.G + t / per_head;
    const int i0 = (i_first + t % per_head) * BR;
    char* dst = smem + QDO_OFF + buf * BUFB;
    qloader.load(dst, a.Q + (si.tok0 * p.Hq + hq) * D, qstride, i0, n - 1, v, lane);
    qloader.load(dst + TILEB, a.dO + (si.tok0 * p.Hq + hq) * D, qstride, i0, n - 1, v, lane);
    if (tid < BR) {
      stat_ok = i0 + tid < n;
      const int r = stat_ok ? i0 + tid : n - 1;
      const long si_ = stat_base + (long)hq * p.lse_head_stride + r;
      lraw = a.LSE[si_];
      draw = a.Dvec[si_];
    }
  };
  auto commit_stats = [&](int buf) {
    if (tid < BR) {
      // rows past the end get L = +inf so that P = exp2(. - inf) = 0 there
      *(float*)(smem + LS_OFF + (buf * BR + tid) * 4) = stat_ok ? lraw * kLog2e : INFINITY;
      *(float*)(smem + DV_OFF + (buf * BR + tid) * 4) = stat_ok ? draw : 0.f;
    }
  };

  // ---- K_j, V_j (Algorithm 2, line 6) stay in LDS for the whole loop
  tile_load_async<D, BC, 8>(smem + KT_OFF, a.K + (si.tok0 * p.Hkv + g) * D, kstride, j0, n - 1, v, lane);
  tile_load_async<D, BC, 8>(smem + VT_OFF, a.V + (si.tok0 * p.Hkv + g) * D, kstride, j0, n - 1, v, lane);
  issue_loads(0, 0);
  wait_vmem();
  commit_stats(0);
  lds_barrier();

  // ---- lane constants of the LDS addressing
  // row operands (rows row0 + lq, row0 a multiple of 32): address = (zrow ^ 32*ks) + row0 * ROWB + tile
  const int zrow = lq * ROWB + 16 * (hh ^ swz<ROWB>(lq));
  // column operands (rows row0 + 4*hh + (p >> 2) + 8*u, row0 a multiple of 16, columns 32*dt..):
  // address = (zcol[u] ^ 64*dt) + row0 * ROWB + tile
  const int p16 = lane & 15, g16 = (lane >> 4) & 1;
  int zcol[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
    zcol[u] = swz_off<ROWB>(4 * hh + (p16 >> 2) + 8 * u, 2 * g16 + ((p16 & 3) >> 1)) + 8 * (p16 & 1);
  const int zk = zrow + 32 * kg * ROWB;  // K_j / V_j row operands of this wavefront

  // ---- dK_j^T, dV_j^T accumulators (line 7): rows = head dim, columns = this wavefront's
  //      32 keys; partial over this wavefront's half of the query rows
  f32x16 dKt[DT], dVt[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dKt[dt] = dVt[dt] = (f32x16){0};

  const int key = j0 + 32 * kg + lq;  // this lane's key column
  const bool key_ok = key < n;

  for (int t = 0; t < nsteps; ++t) {
    const int buf = t & 1;
    const int i0 = (i_first + t % per_head) * BR;
    if (t + 1 < nsteps) issue_loads(t + 1, buf ^ 1);
    const int qoff = QDO_OFF + buf * BUFB;  // this step's Q_i tile; dO_i follows at + TILEB
    const int zq = zrow + qoff, zc0 = zcol[0] + qoff, zc1 = zcol[1] + qoff;
    const int stat_off = buf * BR * 4;

#pragma unroll
    for (int tq = 0; tq < QTW; ++tq) {
      const int qtile = qh * QTW + tq;
      const int r0 = i0 + 32 * qtile;  // first query row of this tile
      // ---- S = Q_i K_j^T (line 10) and dP = dO_i V_j^T (line 13)
      f32x16 S = {0}, dP = {0};
      const int qrow = 32 * qtile * ROWB;
      mfma_stream<2 * KS, 3, 2>(
          [&](int i) {
            const int x = 32 * (i >> 1);
            return OperandPair{lds_b128(smem, (zq ^ x) + qrow + (i & 1) * TILEB),
                               lds_b128(smem, (zk ^ x) + ((i & 1) ? VT_OFF : KT_OFF))};
          },
          [&](int i, const OperandPair& o) {
            if (i & 1) dP = mfma32(o.a, o.b, dP);
            else S = mfma32(o.a, o.b, S);
          });
      // ---- P = exp(S - L) (line 11), dS = P o (dP - D) (line 14)
      const bool need_mask = (CAUSAL && j0 + 32 * kg + 31 > r0) || (j0 + BC > n);
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 Lv = *(const f32x4*)(smem + LS_OFF + stat_off + (32 * qtile + 8 * r4 + 4 * hh) * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) S[4 * r4 + u] = fast_exp2(__builtin_fmaf(S[4 * r4 + u], c2, -Lv[u]));
      }
      if (need_mask) {  // tiles on the diagonal or at the end of the sequence only
        asm volatile("; keep this a branch: the mask costs three instructions per element" ::);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const bool vis = key_ok && (!CAUSAL || key <= r0 + acc_row(r, hh));
          if (!vis) S[r] = 0.f;
        }
      }
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 Dv = *(const f32x4*)(smem + DV_OFF + stat_off + (32 * qtile + 8 * r4 + 4 * hh) * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) dP[4 * r4 + u] = S[4 * r4 + u] * (dP[4 * r4 + u] - Dv[u]);
      }
      bf16x8 Pf[2], dSf[2];
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        Pf[s2] = pack8(S, s2);
        dSf[s2] = pack8(dP, s2);
      }
      // ---- dV_j^T += dO_i^T P (line 12), dK_j^T += Q_i^T dS (line 16)
      mfma_stream<4 * DT, 4, 2>(
          [&](int i) {
            const int dt = i >> 2, s2 = (i >> 1) & 1;
            const int ro = (32 * qtile + 16 * s2) * ROWB + (i & 1) * TILEB;
            return lds_tr_pair(smem, (zc0 ^ (64 * dt)) + ro, (zc1 ^ (64 * dt)) + ro);
          },
          [&](int i, bf16x8 x) {
            const int dt = i >> 2, s2 = (i >> 1) & 1;
            if (i & 1) dVt[dt] = mfma32(x, Pf[s2], dVt[dt]);
            else dKt[dt] = mfma32(x, dSf[s2], dKt[dt]);
          });
    }
    // the next step's tiles and statistics were requested before this step's compute
    wait_vmem();
    commit_stats(buf ^ 1);
    lds_barrier();  // next tiles visible; nobody reads this step's Q_i / dO_i any more
  }

  // ---- combine the two query halves and write dK_j, dV_j (line 18); dK carries the scaling
  float* red = (float*)(smem + QDO_OFF);  // 4 * DT * 16 * 64 floats <= 64 KiB, free after the loop
  const float sc = p.scale;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    f32x16* accs = which == 0 ? dKt : dVt;
    if (qh == 1) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[((kg * DT + dt) * 16 + r) * 64 + lane] = accs[dt][r];
    }
    __syncthreads();
    if (qh == 0 && key_ok) {
      __bf16* dst = (which == 0 ? a.dK : a.dV) + ((si.tok0 + key) * p.Hkv + g) * D + 4 * hh;
      const float mul = which == 0 ? sc : 1.f;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          float x[4];
#pragma unroll
          for (int u = 0; u < 4; ++u)
            x[u] = (accs[dt][4 * r4 + u] + red[((kg * DT + dt) * 16 + 4 * r4 + u) * 64 + lane]) * mul;
          u32x2 o;
          o[0] = pack_bf16(x[0], x[1]);
          o[1] = pack_bf16(x[2], x[3]);
          *(u32x2*)(dst + 32 * dt + 8 * r4) = o;
        }
    }
    __syncthreads();
  }
}

// dQ kernel: 8 wavefronts, each owning 32 whole query rows of a 256-row block. Same phase
// structure as the forward kernel: a matrix phase (S^T, dP^T of block j and the dQ^T update
// with block j - 1) and a vector phase (P and dS of block j), the two wave groups one phase
// apart, K_j / V_j tiles streaming HBM -> LDS two blocks ahead into a ring of four buffers.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(512) void bwd_dq_kernel(BwdArgs a) {
  constexpr int BR = 256, BC = 64, RING = 4;
  constexpr int KS = D / 16, DT = D / 32;
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = BC * ROWB, BUFB = 2 * TILEB;  // one buffer = K_j | V_j

  __shared__ __attribute__((aligned(1024))) char smem[RING * BUFB];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = w >> 2;  // 0: matrix phase on even phases, 1: on odd phases
  const int lq = lane & 31, hh = lane >> 5;
  const int nblk = (p.N + BR - 1) / BR;
  const BlockCoord bc = block_coord<CAUSAL>(nblk, p.Hq, p.nseq);
  if (!bc.valid) return;
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

  // ---- Q_i, dO_i operands and L_i, D_i of this lane's query row: registers for the whole kernel
  const int wrow0 = i0 + 32 * w;
  const int row = wrow0 + lq;
  const int rowc = row < n ? row : n - 1;
  bf16x8 Qf[KS], dOf[KS];
  {
    const __bf16* qp = a.Q + ((si.tok0 + rowc) * p.Hq + h) * D + 8 * hh;
    const __bf16* gp = a.dO + ((si.tok0 + rowc) * p.Hq + h) * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Qf[ks] = *(const bf16x8*)(qp + 16 * ks);
      dOf[ks] = *(const bf16x8*)(gp + 16 * ks);
    }
  }
  const long stat = s * p.lse_seq_stride + (long)h * p.lse_head_stride + (p.cu_seqlens ? si.tok0 : 0) + rowc;
  const float Lq = row < n ? a.LSE[stat] * kLog2e : INFINITY;  // rows past the end: P = 0
  const float Dq = a.Dvec[stat];

  f32x16 dQt[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dQt[dt] = (f32x16){0};

  const int ncol_all = (n + BC - 1) / BC;
  int ncol = ncol_all;
  if (CAUSAL) {
    const int last_row = (i0 + BR < n ? i0 + BR : n) - 1;
    const int c = last_row / BC + 1;
    ncol = c < ncol_all ? c : ncol_all;
  }

  // tile copies: group 1 brings in the K tiles, group 0 the V tiles, each at the start of its
  // own vector phase (see the forward kernel)
  TileLoader<D, BC, 4> loader;
  loader.init(kstride, w & 3, lane);
  constexpr int TPW = TileLoader<D, BC, 4>::PER;
  auto issue_tile = [&](int j) {
    char* dst = smem + (j % RING) * BUFB + (grp == 0 ? TILEB : 0);
    loader.load(dst, grp == 0 ? Vb : Kb, kstride, j * BC, n - 1, w & 3, lane);
  };
  issue_tile(0);
  issue_tile(1);
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    touch(Qf[ks]);
    touch(dOf[ks]);
  }
  touch(Lq);
  touch(Dq);
  wait_vmem();
  lds_barrier();

  const int zrow = lq * ROWB + 16 * (hh ^ swz<ROWB>(lq));
  const int p16 = lane & 15, g16 = (lane >> 4) & 1;
  int zcol[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
    zcol[u] = swz_off<ROWB>(4 * hh + (p16 >> 2) + 8 * u, 2 * g16 + ((p16 & 3) >> 1)) + 8 * (p16 & 1);

  const float c2 = p.scale_log2e;
  const int wrow_last = wrow0 + 31;
  const int lim_row = CAUSAL ? (row < n - 1 ? row : n - 1) : n - 1;  // last visible column of this lane's row

  f32x16 S[2], dP[2];
  bf16x8 dSf[2][2];

  // ================= matrix phase j =================
  auto matrix_phase = [&](int j) {
    __builtin_amdgcn_s_setprio(2);
    if (j < ncol && (!CAUSAL || j * BC <= wrow_last)) {
      // ---- S^T = K_j Q_i^T (line 10), dP^T = V_j dO_i^T (line 13)
      const int zk = zrow + (j % RING) * BUFB;
      S[0] = S[1] = dP[0] = dP[1] = (f32x16){0};
      mfma_stream<4 * KS, 4, 1>(
          [&](int i) {
            const int ks = i >> 2, kt = (i >> 1) & 1;
            return lds_b128(smem, (zk ^ (32 * ks)) + 32 * kt * ROWB + (i & 1) * TILEB);
          },
          [&](int i, bf16x8 x) {
            const int ks = i >> 2, kt = (i >> 1) & 1;
            if (i & 1) dP[kt] = mfma32(x, dOf[ks], dP[kt]);
            else S[kt] = mfma32(x, Qf[ks], S[kt]);
          });
    }
    if (j >= 1 && (!CAUSAL || (j - 1) * BC <= wrow_last)) {
      // ---- dQ_i^T += K_{j-1}^T dS^T (line 15)
      const int kb = ((j - 1) % RING) * BUFB;
      const int zc0 = zcol[0] + kb, zc1 = zcol[1] + kb;
      mfma_stream<4 * DT, 3, 2>(
          [&](int i) {
            const int dt = i >> 2, ro = (16 * (i & 3)) * ROWB;
            return lds_tr_pair(smem, (zc0 ^ (64 * dt)) + ro, (zc1 ^ (64 * dt)) + ro);
          },
          [&](int i, bf16x8 x) { dQt[i >> 2] = mfma32(x, dSf[(i >> 1) & 1][i & 1], dQt[i >> 2]); });
    }
    __builtin_amdgcn_s_setprio(0);
  };

  // ================= vector phase j: P = exp(S - L) (line 11), dS = P o (dP - D) (line 14) =================
  auto vector_phase = [&](int j) {
    if (j >= ncol || (CAUSAL && j * BC > wrow_last)) return;
    const int col0 = j * BC;
    const bool need_mask = (CAUSAL && col0 + BC - 1 > wrow0) || (col0 + BC > n);
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) S[kt][r] = fast_exp2(__builtin_fmaf(S[kt][r], c2, -Lq));
      if (need_mask) {  // tiles on the diagonal or at the end of the sequence only
        asm volatile("; keep this a branch: the mask costs three instructions per element" ::);
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (col0 + 32 * kt + acc_row(r, hh) > lim_row) S[kt][r] = 0.f;
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) dP[kt][r] = S[kt][r] * (dP[kt][r] - Dq);
      dSf[kt][0] = pack8(dP[kt], 0);
      dSf[kt][1] = pack8(dP[kt], 1);
    }
  };

  // phases: see the forward kernel
  if (grp == 0) {
    for (int j = 0; j <= ncol; ++j) {
      matrix_phase(j);
      lds_barrier();
      issue_tile(j + 2);
      vector_phase(j);
      wait_vmem_upto<TPW>();
      lds_barrier();
    }
  } else {
    issue_tile(2);
    lds_barrier();
    for (int j = 0; j <= ncol; ++j) {
      matrix_phase(j);
      wait_vmem_upto<TPW>();
      lds_barrier();
      if (j < ncol) {
        issue_tile(j + 3);
        vector_phase(j);
        lds_barrier();
      }
    }
  }

  if (row < n) {
    __bf16* op = a.dQ + ((si.tok0 + row) * p.Hq + h) * D + 4 * hh;
    const float sc = p.scale;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 o;
        o[0] = pack_bf16(dQt[dt][4 * r4 + 0] * sc, dQt[dt][4 * r4 + 1] * sc);
        o[1] = pack_bf16(dQt[dt][4 * r4 + 2] * sc, dQt[dt][4 * r4 + 3] * sc);
        *(u32x2*)(op + 32 * dt + 8 * r4) = o;
      }
  }
}

template <int D>
static hipError_t launch_bwd_d(const BwdArgs& a, int causal, int stages, hipStream_t st) {
  const long nrows = (long)a.p.total_tokens * a.p.Hq;
  constexpr int RPB = 256 / (D / 8);
  hipError_t e = hipSuccess;
  if (stages & 1) {
    hipLaunchKernelGGL((bwd_prep_kernel<D>), dim3((unsigned)((nrows + RPB - 1) / RPB)), dim3(256), 0, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (stages & 2) {
    dim3 grid(grid_size((a.p.N + 127) / 128, a.p.Hkv * a.p.nseq));
    if (causal) hipLaunchKernelGGL((bwd_dkdv_kernel<D, true>), grid, dim3(512), 0, st, a);
    else hipLaunchKernelGGL((bwd_dkdv_kernel<D, false>), grid, dim3(512), 0, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (stages & 4) {
    dim3 grid(grid_size((a.p.N + 255) / 256, a.p.Hq * a.p.nseq));
    if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true>), grid, dim3(512), 0, st, a);
    else hipLaunchKernelGGL((bwd_dq_kernel<D, false>), grid, dim3(512), 0, st, a);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_bwd(const BwdArgs& a, int d, int causal, int stages, hipStream_t st) {
  if (d == 64) return launch_bwd_d<64>(a, causal, stages, st);
  return launch_bwd_d<128>(a, causal, stages, st);
}

}  // namespace fa
