// Backward pass of exact attention for gfx950 (Algorithm 2 of the paper).
//
// Three launches on the caller's stream (the plain full backward folds the first into the
// third, which then runs before the second: two launches, see OWN_D):
//   1. prep:  D = rowsum(dO o O) (Algorithm 2, line 4)
//   2. dK/dV: one workgroup per block of 256 keys of one (sequence, key/value head)
//             (section 3.2 "Backward pass"); it loops over the query heads that share the
//             key/value head and over the row blocks i, recomputes P from the saved
//             logsumexp (line 11) and keeps dK_j, dV_j in MFMA accumulators for the whole
//             loop (lines 12-16 without line 15)
//   3. dQ:    one workgroup per block of 256 query rows; it loops over the column blocks,
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

template <int D, bool F16>
__global__ __launch_bounds__(256) void bwd_prep_kernel(BwdArgs a) {
  constexpr int LPR = D / 8;  // lanes per row, 8 elements each
  constexpr int RPB = 256 / LPR;
  const long nrows = (long)a.p.total_tokens * a.p.Hq;
  const long row = (long)blockIdx.x * RPB + threadIdx.x / LPR;
  const int c = threadIdx.x % LPR;
  const int dh = a.p.d;  // row length in memory, at most D
  float acc = 0.f;
  if (row < nrows && 8 * c < dh) {
    bf16x8 o = *(const bf16x8*)(a.O + row * dh + 8 * c);
    bf16x8 g = *(const bf16x8*)(a.dO + row * dh + 8 * c);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc += widen<F16>(o, t) * widen<F16>(g, t);
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (row < nrows && c == 0) {
    long tok = row / a.p.Hq;
    int h = (int)(row - tok * a.p.Hq);
    a.Dvec[stat_index(a.p, tok, h)] = acc;
  }
}


// dK/dV kernel: 8 wavefronts in two groups of four. Two forms share the code below.
// WIDE (the plain, half precision and padded instantiations): 256 keys per workgroup, wavefront
// v owns keys 32*v.. and visits every tile; see the comment at `if constexpr (WIDE)`.
// Otherwise (dropout, mask: their extra registers leave no room for K_j in registers, and K_j
// plus V_j of 256 keys do not fit in LDS): 128 keys per workgroup, wavefront (kg, grp) owns
// keys 32*kg.. of the column block; the groups take the 32*QTW-row query tiles alternately
// (group = tile index mod 2) and accumulate partial dK_j^T, dV_j^T over their own tiles.
// The description that follows is that of the second form; the first differs in who visits
// which tile and in the ring depth, not in the phases.
//
// Phases. Tile T passes through three stages, one per global phase, a workgroup barrier
// after every phase:
//   phase T     M : S = Q_i K_j^T (line 10) and dP = dO_i V_j^T (line 13)          [MFMA]
//   phase T + 1 V : P = exp(S - L) (line 11), dS = P o (dP - D) (line 14)           [vector ALU]
//   phase T + 2 M': dV_j^T += dO_i^T P (line 12), dK_j^T += Q_i^T dS (line 16)      [MFMA]
// so in phase F the group F mod 2 is in its matrix phase (M' of tile F - 2, then M of tile F)
// while the other group is in its vector phase (V of tile F - 1): the two wavefronts of a
// SIMD alternate between the matrix pipe and the vector ALU.
//
// Q_i | dO_i tiles live in a ring of 5 LDS slots shared by the groups: tile T is read in
// phases T and T + 2, its slot is refilled with tile T + 5, requested at the start of the
// vector phase F = T + 3 (by the group in that phase, so the copy instructions do not hold up
// the matrix pipe) and complete before the barrier that ends phase F + 1.
//
// LDS addressing. Every tile is swizzled (see swz<>). Because the XOR only touches
// address bits 4..7 while row offsets live in bits >= 7/8, the address of every MFMA
// operand is (lane constant) ^ (compile-time constant) + (immediate): the lane
// constants are a handful of registers computed once, instead of one register per
// distinct operand.
constexpr int kDkdvAhead = 4;  // how many MFMAs ahead the LDS operands are requested (3 where K_j takes the registers)
// keys per workgroup of the dK/dV kernel instantiation (the launch needs it for the grid)
constexpr bool dkdv_wide(int D, bool dropout, bool mask) { return !dropout && !mask; }
constexpr int dkdv_block_keys(int D, bool dropout, bool mask) { return dkdv_wide(D, dropout, mask) ? 256 : 128; }
//
// PAD: head dimension p.d below the tile width D, rows padded with zeros on chip (see the
// forward kernel); only the first p.d columns of dK, dV are stored.
//
// MASK: a tensor M is added to the scaled scores (section 2.2, footnote). Here a lane holds one
// key column and 16 query rows of a tile, and the LDS block is full, so each lane fetches its
// 16 entries of M straight into registers, one tile ahead: requested at the end of the vector
// phase before, complete at the wait that ends the matrix phase in between. The operand
// prefetch distance is halved to make room for them.
//
// LOCAL: sliding window (see the forward kernel). The workgroup visits only the row tiles whose
// window reaches its 256 keys, a wavefront computes only on those that reach its own 32 keys
// (leading and trailing tiles are sat out), and the element mask is applied on the tiles that
// straddle an edge of the band.
//
// DH (PAD only): the head dimension rounded up to a multiple of 32; the products run over the
// first DH columns of the D-wide tiles only (see the forward kernel).
template <int D, bool CAUSAL, bool F16, bool DROPOUT = false, bool PAD = false, bool MASK = false, bool LOCAL = false,
          int DH = D>
__global__ __launch_bounds__(512) void bwd_dkdv_kernel(BwdArgs a) {
  static_assert(DH == D || (PAD && DH % 32 == 0 && DH < D), "a narrower product width is for padded head dimensions");
  static_assert(!MASK || (!DROPOUT && !PAD), "the mask variant is built for the plain kernel");
  static_assert(!LOCAL || (!CAUSAL && !DROPOUT && !PAD && !MASK), "the window variant is built for the plain kernel");
  constexpr bool KREG = !MASK && !DROPOUT;  // K_j operands of the wavefront's 32 keys in registers
  constexpr bool VREG = D == 64 && !MASK && !DROPOUT;  // at d = 64 V_j's as well
  constexpr bool WIDE = dkdv_wide(D, DROPOUT, MASK);
  constexpr int BC = dkdv_block_keys(D, DROPOUT, MASK);  // keys per workgroup
  constexpr int QTW = D == 128 ? 1 : 2;  // 32-row query tiles per wavefront per step
  constexpr int BR = 32 * QTW;          // query rows of one tile
  constexpr int KS = DH / 16, DT = DH / 32;
  constexpr int ROWB = 2 * D;           // row bytes of the Q_i, dO_i, K_j, V_j tiles
  constexpr int RING = WIDE ? 4 : 5;
  // byte offsets inside the LDS block (WIDE: K_j never enters LDS, V_j only when it is not in registers)
  constexpr bool K_IN_LDS = !WIDE, V_IN_LDS = !(WIDE && VREG);
  constexpr int KT_OFF = 0, VT_OFF = K_IN_LDS ? BC * ROWB : 0, QDO_OFF = VT_OFF + (V_IN_LDS ? BC * ROWB : 0);
  constexpr int TILEB = BR * ROWB, BUFB = 2 * TILEB;  // one Q_i (or dO_i) tile; one ring slot = Q_i | dO_i
  constexpr int LS_OFF = QDO_OFF + RING * BUFB;       // [slot][row] floats
  constexpr int DV_OFF = LS_OFF + RING * BR * 4;
  constexpr int BITS_OFF = DV_OFF + RING * BR * 4;  // LOCAL: one activity bitmap per wavefront (over the tiles in its range)
  constexpr int LIST_OFF = BITS_OFF + 8 * 8 * kPatternWords;  // LOCAL: the tiles the workgroup visits, four bytes each
  constexpr int SMEM = LOCAL ? LIST_OFF + 4 * 64 * kPatternWords : BITS_OFF;
  static_assert(VT_OFF + BC * ROWB <= 65536 && BUFB <= 32768, "immediate offsets must fit 16 bits");
  static_assert(WIDE || 4 * DT * 16 * 64 * 4 <= RING * BUFB, "the final reduction reuses the ring");
  static_assert(SMEM <= 160 * 1024, "LDS of one compute unit");

  __shared__ __attribute__((aligned(1024))) char smem[SMEM];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int v = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = v & 3, grp = v >> 2;
  const int kgi = WIDE ? v : kg;  // which 32 keys of the block this wavefront owns
  const int gtid = tid & 255;  // thread index inside the group
  const int lq = lane & 31, hh = lane >> 5;
  const BlockCoord bc = block_coord<CAUSAL>((p.Nk + BC - 1) / BC, p.Hkv, p.nseq);  // causal: block 0 is the longest
  if (!bc.valid) return;
  const int g = bc.head, s = bc.seq;
  const SeqInfo si = seq_info(p, s);
  const int n = si.n, nk = si.nk;  // query rows, key rows
  const int off = nk - n;          // position of query 0 among the keys (causal alignment)
  // Causal: a key block's work grows with the number of rows below it, so the launch order (block 0
  // first) is the longest-first order when block indices count from the END of the longest possible
  // sequence: a shorter sequence of a ragged batch owns the last of them, and its blocks are handed out
  // among the equally long remainders of the longer ones instead of ahead of them.
  const int jblk = CAUSAL ? bc.blk - ((p.Nk + BC - 1) / BC - (nk + BC - 1) / BC) : bc.blk;
  if (jblk < 0) return;
  const int j0 = jblk * BC;
  if (j0 >= nk) return;
  const int dh = PAD ? p.d : D;  // row length in memory
  const long qstride = (long)p.Hq * dh, kstride = (long)p.Hkv * dh;
  if (PAD) lds_zero<512>(smem, SMEM);

  const float c2 = p.scale_log2e;
  const int nrt = (n + BR - 1) / BR;         // row tiles of the sequence
  // row tiles entirely above the diagonal are skipped; past the last row tile there is nothing to do
  const int wl = LOCAL ? p.win_left : -1, wr = LOCAL ? p.win_right : -1;  // window bounds (negative: none)
  int i_first = CAUSAL && j0 > off ? (j0 - off) / BR : 0;
  if (LOCAL && wr >= 0 && j0 > off + wr) i_first = (j0 - off - wr) / BR;  // the first row whose window reaches key j0
  if (i_first > nrt) i_first = nrt;
  int i_end = nrt;  // (window: one past the last row tile whose rows still see the block's last key)
  if (LOCAL && wl >= 0) {
    const long last_row = (long)j0 + BC - 1 - off + wl;
    if (last_row / BR + 1 < i_end) i_end = (int)(last_row / BR) + 1;
    if (i_end < i_first) i_end = i_first;
  }
  const int T = (i_end - i_first) * p.G;     // tiles this workgroup visits, over the group's query heads
  const long stat_base = s * p.lse_seq_stride + (p.cu_seqlens ? si.tok0 : 0);

  // Position of a tile in the visiting order: row tile, query head, ring slot, and where the
  // tile starts in Q / dO (elements) and in L / D. Advancing is a few scalar additions. The
  // query heads of the group are the inner loop: their rows of one token are neighbours in
  // memory, and under the mask the tiles above a wavefront's keys then come first, all together.
  struct Cursor {
    int hq, it, slot;
    long qoff, soff;
  };
  const int hq_end = (g + 1) * p.G;
  const long wrap_q = BR * qstride - (long)p.G * dh;  // last head of a row tile -> first head of the next
  const long wrap_s = BR - (long)p.G * p.lse_head_stride;
  auto advance = [&](Cursor& c, int steps) {
    for (int k = 0; k < steps; ++k) {
      ++c.hq;
      c.qoff += dh;
      c.soff += p.lse_head_stride;
      if (c.hq == hq_end) {
        c.hq = g * p.G;
        ++c.it;
        c.qoff += wrap_q;
        c.soff += wrap_s;
      }
      c.slot = c.slot + 1 == RING ? 0 : c.slot + 1;
    }
  };
  const Cursor tile0 = {g * p.G, i_first, 0, ((si.tok0 + (long)i_first * BR) * p.Hq + g * p.G) * dh,
                        stat_base + (long)g * p.G * p.lse_head_stride + (long)i_first * BR};
  // (an entry of the visit list below: the tile's number in that order, and its row tile in the upper half)
  auto cursor_at = [&](unsigned entry, int slot) {
    const int tt = entry & 0xffff, it = entry >> 16, hq = g * p.G + tt - (it - i_first) * p.G;
    return Cursor{hq, it, slot, ((si.tok0 + (long)it * BR) * p.Hq + hq) * dh,
                  stat_base + (long)hq * p.lse_head_stride + (long)it * BR};
  };

  // (256 keys per workgroup) Leading tiles in which every score of THIS wavefront's 32 keys is
  // masked (its keys lie above the tile's last row, or past the end of the sequence), and under a
  // window trailing ones: the wavefront only keeps up with the copies and the barriers.
  int skip = 0, t_stop = T;  // this wavefront computes on tiles skip .. t_stop - 1
  if (j0 + 32 * kgi >= nk) skip = T;
  else if ((CAUSAL || wr >= 0) && j0 + 32 * kgi > off + (LOCAL ? wr : 0)) {
    const int first_useful = (j0 + 32 * kgi - off - (LOCAL ? wr : 0)) / BR;  // first row tile that reaches this wavefront's keys
    skip = (first_useful - i_first) * p.G < T ? (first_useful - i_first) * p.G : T;
  }
  if (LOCAL && wl >= 0) {  // one past the last row tile whose rows still see this wavefront's last key
    const long last_row = (long)j0 + 32 * kgi + 31 - off + wl;
    const long stop = (last_row / BR + 1 - i_first) * p.G;
    if (stop < t_stop) t_stop = (int)stop;
  }
  if (t_stop < skip) t_stop = skip;

  // Block-sparse pattern: whether this wavefront has anything to do on tile t (row tile
  // i_first + t / G of query head g G + t % G; its rows lie in one row block of the pattern, its 32
  // keys in one key block; t inside skip .. t_stop) is one bit of the wavefront's bitmap, gathered
  // here for every t. The workgroup then visits only the tiles that some wavefront has a bit for:
  // every wavefront compacts the union of the eight bitmaps into the same list, so neither copies
  // nor phases are spent on a tile that the pattern removes from all 256 keys.
  const bool sparse = LOCAL && p.bmask != nullptr;
  const unsigned* visit = (const unsigned*)(smem + LIST_OFF);
  int Tv = T;  // tiles the workgroup visits
  bool listed = false;  // the visit follows the list
  if (LOCAL && sparse) {
    unsigned long long* bits = (unsigned long long*)(smem + BITS_OFF) + v * kPatternWords;
    const uint8_t* bm0 = p.bmask + s * p.bmask_bs + (long)((j0 + 32 * kgi < nk ? j0 + 32 * kgi : nk - 1) >> p.bmask_log2);
    for (int q = 0; q * 64 < T; q += 4) {  // (four words a round: their loads are in flight together)
      uint8_t b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int tt = (q + u) * 64 + lane;
        const int it = i_first + tt / p.G, hq = g * p.G + tt % p.G;
        b[u] = tt >= skip && tt < t_stop ? bm0[hq * p.bmask_hs + (long)((it * BR) >> p.bmask_log2) * p.bmask_cols] : 0;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const unsigned long long m = __builtin_amdgcn_ballot_w64(b[u] != 0);
        if (lane == 0 && (q + u) * 64 < T) bits[q + u] = m;
      }
    }
    lds_barrier();
    const unsigned long long* all_bits = (const unsigned long long*)(smem + BITS_OFF);
    int cnt = 0;
    for (int q = 0; q * 64 < T; ++q) {
      unsigned long long u = 0;
#pragma unroll
      for (int ww = 0; ww < 8; ++ww) u |= all_bits[ww * kPatternWords + q];
      const bool on = ((u >> lane) & 1) != 0;
      const unsigned long long m64 = __builtin_amdgcn_ballot_w64(on);
      const int before = __builtin_amdgcn_mbcnt_hi((unsigned)(m64 >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m64, 0u));
      const int tt = q * 64 + lane;
      if (on) ((unsigned*)visit)[cnt + before] = (unsigned)tt | ((unsigned)(i_first + tt / p.G) << 16);  // (all eight wavefronts write the same list)
      cnt += __builtin_popcountll(m64);
    }
    // (a visit that the list would shorten by less than half stays the plain one: see the forward kernel)
    listed = 2 * cnt <= T;
    if (listed) Tv = cnt;
  }
  // The list entry of the tile at position t of the visit (past its end: the last one). Lane l keeps
  // entry win_base + l, so that a lookup is a lane read; step t asks for positions t .. t + 3.
  int win_base = 0;
  unsigned win = LOCAL && listed ? visit[lane] : 0u;
  auto tile_no = [&](int t) {
    if (!(LOCAL && listed)) return (unsigned)t;
    const int tc = t < Tv ? t : Tv - 1;
    if (tc < 0) return 0u;
    if ((unsigned)(tc - win_base) >= 64u) {
      win_base = tc < 8 ? 0 : tc - 8;
      const int e = win_base + lane;
      win = visit[e < 64 * kPatternWords ? e : 64 * kPatternWords - 1];
    }
    return (unsigned)__builtin_amdgcn_readlane(win, tc - win_base);
  };

  // Q_i, dO_i (line 9) go HBM -> LDS directly; L_i, D_i travel through two registers of the
  // issuing group's first BR threads. The raw statistics are only touched (scaled, masked)
  // when they are committed to LDS: using them earlier would make the compiler wait for
  // them, and with them for the copies in flight.
  float lraw = 0.f, draw = 0.f;
  bool stat_ok = false;
  TileLoader<D, BR, 4, PAD> qloader;  // Q_i and dO_i tiles have the same shape and row pitch
  qloader.init(qstride, kg, lane, dh / 8);
  auto issue_loads = [&](const Cursor& c) {
    char* dst = smem + QDO_OFF + c.slot * BUFB;
    if ((c.it + 1) * BR <= n) {  // all rows exist
      qloader.load_at(dst, a.Q + c.qoff, kg);
      qloader.load_at(dst + TILEB, a.dO + c.qoff, kg);
      if (gtid < BR) {
        stat_ok = true;
        lraw = (a.LSE + c.soff)[gtid];
        draw = (a.Dvec + c.soff)[gtid];
      }
    } else {  // the last rows of the sequence: rows past the end repeat row n - 1
      const int i0 = c.it * BR;
      const long first = c.qoff - (long)i0 * qstride;  // row 0 of this head
      tile_load_async<D, BR, 4, PAD>(dst, a.Q + first, qstride, i0, n - 1, kg, lane, dh / 8);
      tile_load_async<D, BR, 4, PAD>(dst + TILEB, a.dO + first, qstride, i0, n - 1, kg, lane, dh / 8);
      if (gtid < BR) {
        stat_ok = i0 + gtid < n;
        const int r = stat_ok ? gtid : n - 1 - i0;
        lraw = (a.LSE + c.soff)[r];
        draw = (a.Dvec + c.soff)[r];
      }
    }
  };
  auto commit_stats = [&](int slot) {
    if (gtid < BR) {
      const int o = (slot * BR + gtid) * 4;
      // L in the exponent's base; rows past the end get L = +inf so that P = exp2(. - inf) = 0.
      // D is stored negated: it is the initial value of the dP accumulator (line 14).
      // (mask: a row left without keys has L = -inf and, like a row past the end, P = 0)
      *(float*)(smem + LS_OFF + o) = stat_ok && !((MASK || LOCAL) && lraw == -INFINITY) ? lraw * kLog2e : INFINITY;
      *(float*)(smem + DV_OFF + o) = stat_ok ? -draw : 0.f;
    }
  };

  // ---- K_j, V_j (Algorithm 2, line 6) are brought into LDS once (their MFMA operands are then
  //      read from there, or from registers, see Kf / Vf below); tiles 0..2 are requested up
  //      front by all wavefronts
  if (K_IN_LDS)
    tile_load_async<D, BC, 8, PAD>(smem + KT_OFF, a.K + (si.tok0k * p.Hkv + g) * dh, kstride, j0, nk - 1, v, lane, dh / 8);
  if (V_IN_LDS)
    tile_load_async<D, BC, 8, PAD>(smem + VT_OFF, a.V + (si.tok0k * p.Hkv + g) * dh, kstride, j0, nk - 1, v, lane, dh / 8);
  // this lane's key column, and (WIDE) its K_j / V_j operands straight from memory: the 8
  // elements 16 ks + 8 hh .. of the key's row are exactly what lane (lq, hh) feeds to MFMA ks
  const int key = j0 + 32 * kgi + lq;
  const bool key_ok = key < nk;
  bf16x8 Kf[KREG ? KS : 1];
  bf16x8 Vf[VREG ? KS : 1];
  if constexpr (WIDE) {
    const long krow = ((si.tok0k + (key_ok ? key : nk - 1)) * p.Hkv + g) * dh + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Kf[ks] = (bf16x8){0};
      if (VREG) Vf[ks] = (bf16x8){0};
      if (!PAD || 16 * ks + 8 * hh < dh) {
        Kf[ks] = *(const bf16x8*)(a.K + krow + 16 * ks);
        if (VREG) Vf[ks] = *(const bf16x8*)(a.V + krow + 16 * ks);
      }
    }
  }
  {
    Cursor c = tile0;
    for (int t = 0; t < (WIDE ? 2 : 3) && t < Tv; ++t) {
      if (LOCAL && listed) c = cursor_at(tile_no(t), t);
      const long first = c.qoff - (long)c.it * BR * qstride;  // row 0 of this head
      char* dst = smem + QDO_OFF + c.slot * BUFB;
      tile_load_async<D, BR, 8, PAD>(dst, a.Q + first, qstride, c.it * BR, n - 1, v, lane, dh / 8);
      tile_load_async<D, BR, 8, PAD>(dst + TILEB, a.dO + first, qstride, c.it * BR, n - 1, v, lane, dh / 8);
      if (tid >= t * BR && tid < (t + 1) * BR) {  // 3 * BR <= 512 threads
        const int row = c.it * BR + tid - t * BR;
        const bool ok = row < n;
        const long si_ = stat_base + (long)c.hq * p.lse_head_stride + (ok ? row : n - 1);
        const float l = a.LSE[si_], dd = a.Dvec[si_];
        const int o = (c.slot * BR + tid - t * BR) * 4;
        *(float*)(smem + LS_OFF + o) = ok && !((MASK || LOCAL) && l == -INFINITY) ? l * kLog2e : INFINITY;
        *(float*)(smem + DV_OFF + o) = ok ? -dd : 0.f;
      }
      advance(c, 1);
    }
  }
  if constexpr (WIDE) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      touch(Kf[ks]);
      if (VREG) touch(Vf[ks]);
    }
  }
  wait_vmem();
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
  const int zk = zrow + 32 * kgi * ROWB;  // K_j / V_j row operands of this wavefront

  // ---- dK_j^T, dV_j^T accumulators (line 7): rows = head dim, columns = this wavefront's
  //      32 keys; partial over this group's tiles
  f32x16 dKt[DT], dVt[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dKt[dt] = dVt[dt] = (f32x16){0};

  f32x16 S[QTW], dP[QTW];
  bf16x8 Pf[QTW][2], dSf[QTW][2];

  // ---- the MFMA work of a tile, as index -> (operand reads, MFMA) maps for mfma_stream_*
  // The S and dP products take both operands from LDS, two 16-byte reads per MFMA: exactly what
  // the LDS port delivers in the time the four SIMDs need for one MFMA each. K_j never changes,
  // so its operands are read once (32 registers at d = 128; the prefetch ring shrinks by one
  // entry to pay for them) and, at d = 64 where there is room, V_j's as well.
  if (KREG && !WIDE) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Kf[ks] = lds_b128(smem, (zk ^ (32 * ks)) + KT_OFF);
  }
  if (VREG && !WIDE) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Vf[ks] = lds_b128(smem, (zk ^ (32 * ks)) + VT_OFF);
  }
  constexpr int NM = QTW * 2 * KS;   // S and dP: 16 MFMAs
  constexpr int NM2 = QTW * 4 * DT;  // dV and dK: 16 MFMAs
  // (mask, window / pattern: a shorter prefetch, their bookkeeping needs the registers)
  constexpr int AH = MASK ? (D == 128 ? 1 : 2) : LOCAL && D == 128 ? 1 : (KREG && D == 128 ? 3 : kDkdvAhead);
  // MASK: this lane's entries of M for the wavefront's next tile (raw 16-bit elements), row by row
  uint32_t mraw[MASK ? QTW * 16 : 1];
  auto issue_mask_loads = [&](const Cursor& c) {
    if constexpr (MASK) {
      const int keyc = key < nk ? key : nk - 1;
      // entry (row, key) of this head's M: a wave-uniform row address plus one per-lane offset
      const char* m0 = (const char*)(p.mask + s * p.mask_bs + c.hq * p.mask_hs);
      if ((c.it + 1) * BR <= n) {  // all rows exist
        unsigned voff = (unsigned)((4 * hh * p.mask_rs + keyc) * 2);
        asm volatile("" : "+v"(voff));  // (recomputed for every tile instead of held in registers)
#pragma unroll
        for (int e = 0; e < QTW * 16; ++e) {
          const char* rowp = m0 + (long)(c.it * BR + 32 * (e / 16) + acc_row(e % 16, 0)) * p.mask_rs * 2;
          mraw[e] = *(const unsigned short*)(rowp + voff);
        }
      } else {  // the last rows of the sequence: rows past the end repeat row n - 1
#pragma unroll
        for (int e = 0; e < QTW * 16; ++e) {
          const int row = c.it * BR + 32 * (e / 16) + acc_row(e % 16, hh);
          mraw[e] = *(const unsigned short*)(m0 + ((long)(row < n ? row : n - 1) * p.mask_rs + keyc) * 2);
        }
      }
    }
  };
  bf16x8 pre[AH];  // first operands of the next M', requested at the end of the vector phase before it
  auto load_m = [&](const Cursor& c, int i) {  // operands of S (even i) and dP (odd i)
    const int tq = i / (2 * KS), k = i % (2 * KS), x = 32 * (k >> 1);
    const int zq = zrow + QDO_OFF + c.slot * BUFB;
    if (k == 1) {
      // dP starts at -D_i, so the products leave dP - D in the accumulator (line 14); read
      // together with the operands of the first dP product
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 Dn = *(const f32x4*)(smem + DV_OFF + c.slot * BR * 4 + (32 * tq + 8 * r4 + 4 * hh) * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) dP[tq][4 * r4 + u] = DROPOUT ? 0.f : Dn[u];  // dropout: see phase_v
      }
      FA_SCHED_DSRD(4);
    }
    const bf16x8 qa = lds_b128(smem, (zq ^ x) + 32 * tq * ROWB + (i & 1) * TILEB);
    if ((i & 1) ? VREG : KREG) return OperandPair{qa, qa};
    return OperandPair{qa, lds_b128(smem, (zk ^ x) + ((i & 1) ? VT_OFF : KT_OFF))};
  };
  auto mma_m = [&](int i, const OperandPair& o) {
    const int tq = i / (2 * KS), k = i % (2 * KS);
    if (k & 1) dP[tq] = mfma32<F16>(o.a, VREG ? Vf[k >> 1] : o.b, dP[tq]);
    else S[tq] = mfma32<F16>(o.a, KREG ? Kf[k >> 1] : o.b, k == 0 ? (f32x16){0} : S[tq]);
  };
  auto load_m2 = [&](const Cursor& c, int i) {  // Q_i^T (even i) or dO_i^T (odd i) operand of dK / dV
    const int tq = i / (4 * DT), k = i % (4 * DT), dt = k >> 2, s2 = (k >> 1) & 1;
    const int qoff = QDO_OFF + c.slot * BUFB + (32 * tq + 16 * s2) * ROWB + (i & 1) * TILEB;
    return lds_tr_pair(smem, ((zcol[0] + qoff) ^ (64 * dt)), ((zcol[1] + qoff) ^ (64 * dt)));
  };
  auto mma_m2 = [&](int i, bf16x8 x) {
    const int tq = i / (4 * DT), k = i % (4 * DT), dt = k >> 2, s2 = (k >> 1) & 1;
    if (i & 1) dVt[dt] = mfma32<F16>(x, Pf[tq][s2], dVt[dt]);
    else dKt[dt] = mfma32<F16>(x, dSf[tq][s2], dKt[dt]);
  };
  auto phase_v = [&](const Cursor& c) {  // P, dS
    const int i0 = c.it * BR;
    const int stat_off = c.slot * BR * 4;
#pragma unroll
    for (int tq = 0; tq < QTW; ++tq) {
      const int r0 = i0 + 32 * tq;  // first query row of this tile
      const bool need_mask = (CAUSAL && j0 + 32 * kgi + 31 > r0 + off) || (j0 + BC > nk) ||
                             (LOCAL && ((wr >= 0 && j0 + 32 * kgi + 31 > r0 + off + wr) ||
                                        (wl >= 0 && j0 + 32 * kgi < r0 + 31 + off - wl)));
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 Lv = *(const f32x4*)(smem + LS_OFF + stat_off + (32 * tq + 8 * r4 + 4 * hh) * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          float sub = -Lv[u];
          if constexpr (MASK)
            sub = __builtin_fmaf(widen_half<F16>(mraw[16 * tq + 4 * r4 + u], false), kLog2e, sub);
          S[tq][4 * r4 + u] = fast_exp2(__builtin_fmaf(S[tq][4 * r4 + u], c2, sub));
        }
      }
      if (need_mask) {  // tiles on the diagonal or at the end of the sequence only
        asm volatile("; keep this a branch: the mask costs two instructions per element" ::);
        // visible: key < nk and (causal) key <= r0 + off + row of the tile, row = acc_row(r, hh)
        // (window: key <= position + win_right and key >= position - win_left)
        const int kc = key_ok ? (CAUSAL ? key - (r0 + off) - 4 * hh : (wr >= 0 ? key - (r0 + off) - 4 * hh - wr : -1)) : 0x7fffffff;
        const int kb = wl >= 0 ? key - (r0 + off) - 4 * hh + wl : 0x7fffffff;
#pragma unroll
        for (int r = 0; r < 16; ++r) S[tq][r] = kc <= acc_row(r, 0) && (!LOCAL || acc_row(r, 0) <= kb) ? S[tq][r] : 0.f;
      }
      if constexpr (DROPOUT) {
        // dP = keep o (dO V^T) / (1 - p), then dS = P o (dP - D) with the true P; afterwards P
        // itself is masked for dV += P_drop^T dO (its 1 / (1 - p) goes into the final scaling)
        const uint32_t hq_key = p.drop_seed ^ (uint32_t)(s * p.Hq + c.hq) * kDropHead;
        const uint32_t base = (uint32_t)(key >> 2) * kDropCol + hq_key;
        const int sh = 8 * (key & 3);
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 Dn = *(const f32x4*)(smem + DV_OFF + stat_off + (32 * tq + 8 * r4 + 4 * hh) * 4);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int e = 4 * r4 + u;
            const uint32_t x = drop_mix(base + (uint32_t)(r0 + acc_row(e, hh)) * kDropRow);
            const bool kept = ((x >> sh) & 255u) >= p.drop_thr;
            const float pe = S[tq][e], dpe = kept ? dP[tq][e] * p.drop_rp : 0.f;
            dP[tq][e] = pe * (dpe + Dn[u]);  // Dn = -D
            S[tq][e] = kept ? pe : 0.f;
          }
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) dP[tq][r] *= S[tq][r];  // dS = P o (dP - D)
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        Pf[tq][s2] = pack8<F16>(S[tq], s2);
        dSf[tq][s2] = pack8<F16>(dP[tq], s2);
      }
    }
  };

  // Phases 0 .. T + 1. This group's matrix phases are tau = grp, grp + 2, ..; each is followed
  // by its vector phase tau + 1. Group 1 idles through phase 0. A matrix phase is one stream
  // of MFMAs, M' of the previous tile running into M of the current one, and the first
  // operand reads of M' are issued at the end of the vector phase before it: the tile they
  // read has been in LDS for two phases, so they need not wait for the barrier.
  Cursor cur = tile0, prev = tile0, ld = tile0;
  int pending = -1;      // ring slot whose statistics wait in lraw / draw
  auto end_matrix_work = [&]() {  // everything of end_matrix_phase but its barrier
    __builtin_amdgcn_s_setprio(0);
    // The copies requested in the last vector phase: complete, then visible. The wait and the
    // touches are unconditional so that the compiler sees no path on which the statistics
    // loads are still in flight when their registers are written again: it would otherwise
    // put a full wait right behind the next tile's copy requests.
    wait_vmem();
    touch(lraw);
    touch(draw);
    if constexpr (MASK) {
#pragma unroll
      for (int e = 0; e < QTW * 16; ++e) touch(mraw[e]);
    }
    if (pending >= 0) {
      commit_stats(pending);
      pending = -1;
    }
  };
  auto end_matrix_phase = [&]() {
    end_matrix_work();
    lds_barrier();
  };
  auto vector_phase = [&](int tau, bool do_v) {  // phase tau + 1, if it exists
    if (tau + 1 > T + 1) return;
    if (tau + 3 < T) {  // the slot of tile tau - 2, free since the last barrier
      issue_loads(ld);
      pending = ld.slot;
      advance(ld, 2);
    }
    if (do_v) {
      phase_v(cur);
      if (MASK && tau + 2 < T) {  // this wavefront's next tile
        Cursor nxt = cur;
        advance(nxt, 2);
        issue_mask_loads(nxt);
      }
      mfma_stream_begin<NM2, AH, 2>(pre, [&](int i) { return load_m2(cur, i); });
    }
    lds_barrier();
  };

  // the two MFMA streams of the steady state as functions of (prev, cur)
  auto fused_stream = [&]() {  // M' of the previous tile running into M of the current one
    __builtin_amdgcn_s_setprio(2);
    OperandPair ring[AH];
#pragma unroll
    for (int i = 0; i < AH; ++i) ring[i].a = pre[i];
    mfma_stream_run<NM2 + NM, AH, 2>(
        ring,
        [&](int i) {
          if (i < NM2) {
            const bf16x8 x = load_m2(prev, i);
            return OperandPair{x, x};
          }
          return load_m(cur, i - NM2);
        },
        [&](int i, const OperandPair& o) {
          if (i < NM2) mma_m2(i, o.a);
          else mma_m(i - NM2, o);
        });
  };

  if constexpr (WIDE) {
    // 256 keys per workgroup: the eight wavefronts own eight different key groups, so every
    // wavefront visits EVERY tile, nothing is left to add up at the end, and each Q_i / dO_i
    // tile is copied once per 256 keys instead of once per 128 (the copy traffic L2 -> LDS
    // costs about as much as the operand reads from LDS). Group 1 runs the same program one
    // phase behind group 0: tile t is in M in phase 2t (group 0) / 2t + 1 (group 1), in V one
    // phase later, in M' two phases later. Phases 0 .. 2T + 1, one barrier each.
    // Copies: group 0 requests tile t + 2 at the start of its vector phase t (phase 2t + 1) into
    // the slot of tile t - 2, whose last reader was group 1's M' in phase 2t - 1; they are
    // complete and visible when the barrier of phase 2t + 2 falls, two phases before group 0
    // reads the tile. A ring of four slots suffices.
    // Of the two barriers per tile only one is executed: group 0's after its vector phase, which
    // is group 1's after its matrix phase. It orders everything that goes through LDS (a tile and its
    // statistics are requested after the barrier that follows their slot's last readers, waited for
    // and committed before the next but one, and first read after that one); the other one only made
    // the two wavefronts of a SIMD change phase together, and without it a matrix phase that ends
    // early runs on into the vector phase (see the forward kernel).
    advance(ld, 2);
    if constexpr (LOCAL) {
      // (the window / pattern instantiation keeps both barriers of a tile: group 1 one phase behind group 0)
      if (grp == 1) lds_barrier();
      // Window and block-sparse pattern: tile by tile, over the tiles the workgroup visits.
      const unsigned long long* bits = (const unsigned long long*)(smem + BITS_OFF) + v * kPatternWords;
      int word_q = -1;
      unsigned long long word = 0;
      auto active = [&](int t) {  // t: a tile's number in the full order
        if (!sparse) return t >= skip && t < t_stop;
        if ((t >> 6) != word_q) {
          word_q = t >> 6;
          word = bits[word_q];
          word = ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)(word >> 32)) << 32) |
                 (unsigned)__builtin_amdgcn_readfirstlane((unsigned)word);
        }
        return ((word >> (t & 63)) & 1) != 0;
      };
      // One loop body for every tile, the steady-state stream of the plain kernel (M' of tile t - 1
      // running into M of tile t) whenever one of the two tiles is active. At the start of a run of
      // active tiles its M' half multiplies by zero operands (P = dS = 0 stand for the inactive
      // tile before), at the end of a run its M half computes scores nobody uses: half a tile of
      // matrix work per end of a run, the price of keeping a single instruction stream (three
      // streams side by side in one loop spill hundreds of registers). Between runs the wavefront
      // only keeps up with the copies and the barriers.
#pragma unroll
      for (int i = 0; i < AH; ++i) pre[i] = (bf16x8){0};
#pragma unroll
      for (int tq = 0; tq < QTW; ++tq) Pf[tq][0] = Pf[tq][1] = dSf[tq][0] = dSf[tq][1] = (bf16x8){0};
      bool was = false;  // the tile visited before this one was active
      auto step = [&](int t, bool now) {  // one tile: this wavefront's share of its two phases
        if (was || now) fused_stream();
        end_matrix_phase();
        if (grp == 0 && t + 2 < Tv) {
          issue_loads(ld);
          pending = ld.slot;
        }
        if (now) {
          phase_v(cur);
          mfma_stream_begin<NM2, AH, 2>(pre, [&](int i) { return load_m2(cur, i); });
        } else if (was) {
#pragma unroll
          for (int tq = 0; tq < QTW; ++tq) Pf[tq][0] = Pf[tq][1] = dSf[tq][0] = dSf[tq][1] = (bf16x8){0};
        }
        lds_barrier();
        prev = cur;
        was = now;
      };
      if (!listed) {
        for (int t = 0; t < Tv; ++t) {
          step(t, active(t));
          advance(ld, 1);
          advance(cur, 1);
        }
      } else {
        // Following the list, the cursors of positions t, t + 1, t + 2 are carried along and one new
        // one (position t + 3) is made per step: by one advance when that tile follows the one before
        // it in the full order, which inside a block of the pattern it does, from scratch otherwise.
        auto follow = [&](const Cursor& from, unsigned from_entry, unsigned entry, int slot) {
          if ((entry & 0xffff) == (from_entry & 0xffff) + 1) {
            Cursor c = from;
            advance(c, 1);
            return c;
          }
          return cursor_at(entry, slot);
        };
        const unsigned e0 = tile_no(0), e1 = tile_no(1);
        unsigned ld_entry = tile_no(2);
        cur = cursor_at(e0, 0);
        Cursor nx = follow(cur, e0, e1, 1);
        ld = follow(nx, e1, ld_entry, 2);
        for (int t = 0; t < Tv; ++t) {
          step(t, active(tile_no(t) & 0xffff));
          const unsigned e3 = tile_no(t + 3);
          const Cursor c3 = follow(ld, ld_entry, e3, (t + 3) % RING);
          cur = nx;
          nx = ld;
          ld = c3;
          ld_entry = e3;
        }
      }
      if (was) {
        __builtin_amdgcn_s_setprio(2);
        mfma_stream_run<NM2, AH, 2>(pre, [&](int i) { return load_m2(prev, i); }, mma_m2);
      }
      end_matrix_phase();
      if (grp == 0) lds_barrier();  // group 1's last phase
    } else {
      // The loops are written out once per group: which of the two barriers a group executes is then
      // fixed in the code (as a run-time condition on both of them the compiler's output failed its own
      // verification, and as lambdas generic in the group the accumulators ended up in memory).
      auto vector_work = [&](int t, bool do_v, bool loads) {  // a vector phase without its barrier
        if (loads && t + 2 < T) {
          issue_loads(ld);
          pending = ld.slot;
          advance(ld, 1);
        }
        if (do_v) {
          phase_v(cur);
          mfma_stream_begin<NM2, AH, 2>(pre, [&](int i) { return load_m2(cur, i); });
        }
      };
      if (grp == 0) {  // barrier after the vector phase; this group requests the tiles
        int t = 0;
        for (; t < skip; ++t) {
          end_matrix_work();
          vector_work(t, false, true);
          lds_barrier();
          advance(cur, 1);
        }
        if (t < T) {
          __builtin_amdgcn_s_setprio(2);
          mfma_stream<NM, AH, 2>([&](int i) { return load_m(cur, i); }, mma_m);
          end_matrix_work();
          vector_work(t, true, true);
          lds_barrier();
          for (++t; t < T; ++t) {
            prev = cur;
            advance(cur, 1);
            fused_stream();
            end_matrix_work();
            vector_work(t, true, true);
            lds_barrier();
          }
          prev = cur;
          __builtin_amdgcn_s_setprio(2);
          mfma_stream_run<NM2, AH, 2>(pre, [&](int i) { return load_m2(prev, i); }, mma_m2);
        }
        end_matrix_work();
        lds_barrier();  // (none was executed for the last matrix phase)
      } else {  // barrier after the matrix phase
        int t = 0;
        for (; t < skip; ++t) {
          end_matrix_phase();
          vector_work(t, false, false);
          advance(cur, 1);
        }
        if (t < T) {
          __builtin_amdgcn_s_setprio(2);
          mfma_stream<NM, AH, 2>([&](int i) { return load_m(cur, i); }, mma_m);
          end_matrix_phase();
          vector_work(t, true, false);
          for (++t; t < T; ++t) {
            prev = cur;
            advance(cur, 1);
            fused_stream();
            end_matrix_phase();
            vector_work(t, true, false);
          }
          prev = cur;
          __builtin_amdgcn_s_setprio(2);
          mfma_stream_run<NM2, AH, 2>(pre, [&](int i) { return load_m2(prev, i); }, mma_m2);
        }
        end_matrix_phase();
      }
    }

    // ---- write dK_j, dV_j (line 18); dK carries the scaling. The ring is idle now (no copy is
    // requested past the last tile): each wavefront stages its rows there and stores whole rows.
    {
      static_assert(RING * BUFB >= 8 * 32 * ROWB, "the ring holds one 32-key tile per wavefront");
      char* stg = smem + QDO_OFF + v * (32 * ROWB);
      const int key0 = j0 + 32 * kgi;
      const long kvoff = ((si.tok0k + key0) * p.Hkv + g) * dh;
      int ln = lane;  // recomputed here: nothing of the staging addresses is to live across the main loop
      asm volatile("" : "+v"(ln));
      store_tiles_via_lds<DT, F16>(stg, dKt, p.scale, a.dK + kvoff, (long)p.Hkv * dh, nk - key0, dh, ln);
      store_tiles_via_lds<DT, F16>(stg, dVt, 1.f, a.dV + kvoff, (long)p.Hkv * dh, nk - key0, dh, ln);
    }
    return;
  }

  advance(cur, grp);
  advance(ld, 3 + grp);  // first refill: tile 3 in phase 1 (group 0), tile 4 in phase 2 (group 1)
  int tau = grp;
  if (grp == 1) lds_barrier();
  // the group's first matrix phase: M only
  const bool have_first = tau < T;
  if (MASK && have_first) issue_mask_loads(cur);
  if (have_first) {
    __builtin_amdgcn_s_setprio(2);
    mfma_stream<NM, AH, 2>([&](int i) { return load_m(cur, i); }, mma_m);
  }
  end_matrix_phase();
  vector_phase(tau, have_first);
  prev = cur;
  advance(cur, 2);
  // steady state: M' of the previous tile, then M of the current one
  for (tau += 2; tau < T; tau += 2) {
    fused_stream();
    end_matrix_phase();
    vector_phase(tau, true);
    prev = cur;
    advance(cur, 2);
  }
  // the last tile's M', then whatever phases remain
  bool have_prev = have_first;
  for (; tau <= T + 1; tau += 2) {
    if (have_prev) {
      __builtin_amdgcn_s_setprio(2);
      mfma_stream_run<NM2, AH, 2>(pre, [&](int i) { return load_m2(prev, i); }, mma_m2);
      have_prev = false;
    }
    end_matrix_phase();
    vector_phase(tau, false);
  }

  // ---- combine the two groups' partial sums and write dK_j, dV_j (line 18); dK carries the scaling
  float* red = (float*)(smem + QDO_OFF);  // 4 * DT * 16 * 64 floats, free after the loop
  const float sc = p.scale;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    f32x16* accs = which == 0 ? dKt : dVt;
    if (grp == 1) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[((kg * DT + dt) * 16 + r) * 64 + lane] = accs[dt][r];
    }
    __syncthreads();
    if (grp == 0 && key_ok) {
      __bf16* dst = (which == 0 ? a.dK : a.dV) + ((si.tok0k + key) * p.Hkv + g) * dh + 4 * hh;
      const float mul = which == 0 ? sc : (DROPOUT ? p.drop_rp : 1.f);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          float x[4];
#pragma unroll
          for (int u = 0; u < 4; ++u)
            x[u] = (accs[dt][4 * r4 + u] + red[((kg * DT + dt) * 16 + 4 * r4 + u) * 64 + lane]) * mul;
          u32x2 o;
          o[0] = pack2<F16>(x[0], x[1]);
          o[1] = pack2<F16>(x[2], x[3]);
          if (!PAD || 32 * dt + 8 * r4 + 4 * hh < dh) *(u32x2*)(dst + 32 * dt + 8 * r4) = o;
        }
    }
    __syncthreads();
  }
}

// dQ kernel: 8 wavefronts, each owning 32 whole query rows of a 256-row block. Same phase
// structure as the forward kernel: a matrix phase (S^T, dP^T of block j and the dQ^T update
// with block j - 1) and a vector phase (P and dS of block j), the two wave groups one phase
// apart, K_j / V_j tiles streaming HBM -> LDS two blocks ahead into a ring of four buffers.
// MASK: the tensor added to the scaled scores reaches the wavefronts as in the forward kernel
// (a private 32 x 64 piece per block, copied HBM -> LDS one vector phase ahead).
// LOCAL: sliding window, as in the forward kernel (only the column blocks inside the band are
// walked; the element mask on the blocks that straddle an edge of it).
// OWN_D: the kernel computes D_i = rowsum(dO_i o O_i) (line 4) of its own rows itself, from the
// dO_i operands it holds anyway and one pass over its O_i rows, and writes it for the dK/dV kernel,
// which then runs after this one: the whole backward without the separate D pre-pass.
// DH (PAD only): the narrower product width of a padded head dimension (see the forward kernel).
template <int D, bool CAUSAL, bool F16, bool DROPOUT = false, bool PAD = false, bool MASK = false, bool LOCAL = false,
          bool OWN_D = false, int DH = D>
__global__ __launch_bounds__(512) void bwd_dq_kernel(BwdArgs a) {
  static_assert(DH == D || (PAD && DH % 32 == 0 && DH < D), "a narrower product width is for padded head dimensions");
  static_assert(!MASK || (!DROPOUT && !PAD), "the mask variant is built for the plain kernel");
  static_assert(!LOCAL || (!CAUSAL && !DROPOUT && !PAD && !MASK), "the window variant is built for the plain kernel");
  constexpr int BR = 256, BC = 64, RING = 4;
  constexpr int KS = DH / 16, DT = DH / 32;
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = BC * ROWB, BUFB = 2 * TILEB;  // one buffer = K_j | V_j
  constexpr int MASKB = 32 * BC * 2;             // one wavefront's piece of M for one block
  constexpr int MPW = MASK ? MASKB / 1024 : 0;  // copies per wavefront per block

  // (LOCAL: behind the ring, one activity bitmap per wavefront and the list of the key blocks that
  // the workgroup visits, as in the forward kernel)
  constexpr int BITSB = 8 * 8 * kPatternWords, LISTB = 2 * 64 * kPatternWords;
  __shared__ __attribute__((aligned(1024))) char smem[RING * BUFB + (MASK ? 8 * MASKB : 0) + (LOCAL ? BITSB + LISTB : 0)];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = w >> 2;  // 0: matrix phase on even phases, 1: on odd phases
  const int lq = lane & 31, hh = lane >> 5;
  const int nblk = (p.N + BR - 1) / BR;
  const BlockCoord bc = block_coord<CAUSAL>(nblk, p.Hq, p.nseq, p.G);
  if (!bc.valid) return;
  const int rowblk = nblk - 1 - bc.blk;  // longest causal rows first
  const int h = bc.head, s = bc.seq;
  const SeqInfo si = seq_info(p, s);
  const int n = si.n, nk = si.nk, off = nk - n;  // query rows, key rows, position of query 0
  const int i0 = rowblk * BR;
  if (i0 >= n || nk == 0) return;  // (a sequence without keys: dQ = 0 comes from keyless_rows_kernel)
  const int g = h / p.G;
  const int dh = PAD ? p.d : D;  // row length in memory
  const long kstride = (long)p.Hkv * dh;
  const __bf16* Kb = a.K + (si.tok0k * p.Hkv + g) * dh;
  const __bf16* Vb = a.V + (si.tok0k * p.Hkv + g) * dh;
  if (PAD) lds_zero<512>(smem, RING * BUFB);

  // ---- Q_i, dO_i operands and L_i, D_i of this lane's query row: registers for the whole kernel
  const int wrow0 = i0 + 32 * w;
  const int row = wrow0 + lq;
  const int rowc = row < n ? row : n - 1;
  bf16x8 Qf[KS], dOf[KS];
  {
    const __bf16* qp = a.Q + ((si.tok0 + rowc) * p.Hq + h) * dh + 8 * hh;
    const __bf16* gp = a.dO + ((si.tok0 + rowc) * p.Hq + h) * dh + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Qf[ks] = dOf[ks] = (bf16x8){0};
      if (!PAD || 16 * ks + 8 * hh < dh) {
        Qf[ks] = *(const bf16x8*)(qp + 16 * ks);
        dOf[ks] = *(const bf16x8*)(gp + 16 * ks);
      }
    }
  }
  const long stat = s * p.lse_seq_stride + (long)h * p.lse_head_stride + (p.cu_seqlens ? si.tok0 : 0) + rowc;
  float Lq = row < n ? a.LSE[stat] * kLog2e : INFINITY;  // rows past the end: P = 0
  if ((MASK || LOCAL) && Lq == -INFINITY) Lq = INFINITY;  // a row that the mask (the pattern) left without keys: P = 0

  f32x16 dQt[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dQt[dt] = (f32x16){0};
  // At d = 64 there are registers to spare and the vector phase is the longer one: sixteen of
  // them hold -D_i as the initial accumulator of the dP products, which saves the subtraction
  // per element (line 14). Not under dropout, where dP is masked before D is subtracted.
  constexpr bool NEGD = D == 64 && !DROPOUT;
  f32x16 negD;  // filled once D_i has arrived, below

  const int ncol_all = (nk + BC - 1) / BC;
  int ncol = ncol_all, jb = 0;  // column blocks jb .. ncol - 1
  const int wl = LOCAL ? p.win_left : -1, wr = LOCAL ? p.win_right : -1;  // window bounds (negative: none)
  if (CAUSAL || wr >= 0) {
    const int last_pos = (i0 + BR < n ? i0 + BR : n) - 1 + off;
    const int c = (last_pos + (LOCAL ? wr : 0)) / BC + 1;
    ncol = c < ncol_all ? c : ncol_all;
  }
  if (LOCAL && wl >= 0 && i0 + off > wl) jb = (i0 + off - wl) / BC;
  if (ncol < jb) ncol = jb;

  // block-sparse pattern: the wavefront's bitmap over the key blocks, and the list of the blocks
  // that any of the eight bitmaps keeps, which is what the workgroup walks (see the forward kernel)
  const unsigned long long* pattern_bits = (const unsigned long long*)(smem + RING * BUFB) + w * kPatternWords;
  const unsigned short* visit = (const unsigned short*)(smem + RING * BUFB + BITSB);
  const bool sparse = LOCAL && p.bmask != nullptr;
  int tb = jb, tend = ncol;  // positions of the walk; position t stands for block t unless the pattern thins the walk
  bool listed = false;       // the walk follows the list
  if (LOCAL && sparse) {
    const int r0 = wrow0 < n ? wrow0 : n - 1;
    const uint8_t* bm_row = p.bmask + s * p.bmask_bs + h * p.bmask_hs + (long)(r0 >> p.bmask_log2) * p.bmask_cols;
    for (int q = jb >> 6; q * 64 < ncol; q += 4) {  // (four words a round: their loads are in flight together)
      uint8_t b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int jj = (q + u) * 64 + lane;
        b[u] = jj < ncol ? bm_row[(jj * BC) >> p.bmask_log2] : 0;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const unsigned long long bits = __builtin_amdgcn_ballot_w64(b[u] != 0);
        if (lane == 0 && (q + u) * 64 < ncol) ((unsigned long long*)pattern_bits)[q + u] = bits;
      }
    }
    lds_barrier();
    const unsigned long long* all_bits = (const unsigned long long*)(smem + RING * BUFB);
    int cnt = 0;
    for (int q = jb >> 6; q * 64 < ncol; ++q) {
      unsigned long long u = 0;
#pragma unroll
      for (int ww = 0; ww < 8; ++ww) u |= all_bits[ww * kPatternWords + q];
      const int jj = q * 64 + lane;
      const bool on = ((u >> lane) & 1) != 0 && jj >= jb && jj < ncol;
      const unsigned long long m64 = __builtin_amdgcn_ballot_w64(on);
      const int before = __builtin_amdgcn_mbcnt_hi((unsigned)(m64 >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m64, 0u));
      if (on) ((unsigned short*)visit)[cnt + before] = (unsigned short)jj;  // (all eight wavefronts write the same list)
      cnt += __builtin_popcountll(m64);
    }
    // (a walk that the list would shorten by less than half stays the plain one: a thinned walk pays
    // for its lookups in every phase, and a block nobody computes on costs little more than its copies)
    listed = 2 * cnt <= ncol - jb;
    if (listed) {
      tb = 0;
      tend = cnt;
    }
  }
  // the block at position t (past the end of the walk: any block; its tiles are copied and never read)
  auto blk = [&](int t) {
    if (!(LOCAL && listed)) return t;
    const int tc = t < tend ? t : tend - 1;
    return tc < 0 ? 0 : __builtin_amdgcn_readfirstlane((int)visit[tc]);
  };

  // tile copies: group 1 brings in the K tiles, group 0 the V tiles, each at the start of its
  // own vector phase (see the forward kernel)
  TileLoader<D, BC, 4, PAD> loader;
  loader.init(kstride, w & 3, lane, dh / 8);
  constexpr int TPW = TileLoader<D, BC, 4, PAD>::PER;
  auto issue_tile = [&](int t) {  // the block at position t of the walk
    char* dst = smem + (t % RING) * BUFB + (grp == 0 ? TILEB : 0);
    loader.load(dst, grp == 0 ? Vb : Kb, kstride, blk(t) * BC, nk - 1, w & 3, lane);
  };
  char* mbuf = smem + RING * BUFB + w * MASKB;
  const __bf16* Mb = MASK ? p.mask + s * p.mask_bs + h * p.mask_hs : nullptr;
  const int nk8 = (nk + 7) & ~7;
  auto issue_mask = [&](int j) {  // see the forward kernel
    if constexpr (MASK) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      int ln = lane;  // hidden from the optimiser: otherwise it keeps all these addresses in registers across the loop
      asm volatile("" : "+v"(ln));
#pragma unroll
      for (int u = 0; u < MPW; ++u) {
        const int r = 8 * u + (ln >> 3);
        const int qr = wrow0 + r < n ? wrow0 + r : n - 1;
        const int c = (ln & 7) ^ (r & 7);
        int col = j * BC + 8 * c;
        col = col < nk8 ? col : 0;
        dma16(Mb + (long)qr * p.mask_rs + col, mbuf + u * 1024);
      }
    }
  };
  issue_tile(tb);
  issue_tile(tb + 1);
  issue_mask(jb);
  // (D after the first tile copies have been requested: summing it waits for O_i, and the copies need not wait with it)
  float Dq;
  if constexpr (OWN_D) {
    // this lane holds half of its row of dO_i (the elements 16 ks + 8 hh ..): the same half of O_i,
    // multiplied and summed, and the other half from the partner lane
    const __bf16* op = a.O + ((si.tok0 + rowc) * p.Hq + h) * dh + 8 * hh;
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      if (!PAD || 16 * ks + 8 * hh < dh) {
        const bf16x8 o = *(const bf16x8*)(op + 16 * ks);
#pragma unroll
        for (int t = 0; t < 8; ++t) part += widen<F16>(o, t) * widen<F16>(dOf[ks], t);
      }
    Dq = sum_with_partner32(part);
    if (row < n && hh == 0) a.Dvec[stat] = Dq;
  } else {
    Dq = a.Dvec[stat];
  }
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    touch(Qf[ks]);
    touch(dOf[ks]);
  }
  touch(Lq);
  touch(Dq);
  wait_vmem();
  lds_barrier();
#pragma unroll
  for (int r = 0; r < 16; ++r) negD[r] = NEGD ? -Dq : 0.f;

  const int zrow = lq * ROWB + 16 * (hh ^ swz<ROWB>(lq));
  const int p16 = lane & 15, g16 = (lane >> 4) & 1;
  int zcol[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
    zcol[u] = swz_off<ROWB>(4 * hh + (p16 >> 2) + 8 * u, 2 * g16 + ((p16 & 3) >> 1)) + 8 * (p16 & 1);

  const float c2 = p.scale_log2e;
  const int wrow_last = wrow0 + 31 + off;  // position of the last row among the keys
  // last and (window) first visible column of this lane's row
  const int lim_row = CAUSAL || wr >= 0 ? (row + off + (LOCAL ? wr : 0) < nk - 1 ? row + off + (LOCAL ? wr : 0) : nk - 1) : nk - 1;
  const int lo_row = wl >= 0 ? row + off - wl : 0;
  int pattern_q = -1;                 // which word of the bitmap `pattern_word` holds
  unsigned long long pattern_word = 0;
  // a block is skipped by a wavefront when every score it would produce is masked
  auto wave_sees = [&](int j) {
    if (CAUSAL) return j * BC <= wrow_last;
    if (LOCAL) {
      if (!((wr < 0 || j * BC <= wrow_last + wr) && (wl < 0 || j * BC + BC - 1 >= wrow0 + off - wl))) return false;
      if (!sparse) return true;
      if ((j >> 6) != pattern_q) {
        pattern_q = j >> 6;
        pattern_word = pattern_bits[pattern_q];
        pattern_word = ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)(pattern_word >> 32)) << 32) |
                       (unsigned)__builtin_amdgcn_readfirstlane((unsigned)pattern_word);
      }
      return ((pattern_word >> (j & 63)) & 1) != 0;
    }
    return true;
  };

  f32x16 S[2], dP[2];
  bf16x8 dSf[2][2];

  // ================= matrix phase j =================
  auto matrix_phase = [&](int t) {
    __builtin_amdgcn_s_setprio(2);
    if (t < tend && wave_sees(blk(t))) {
      // ---- S^T = K_j Q_i^T (line 10), dP^T = V_j dO_i^T (line 13)
      const int zk = zrow + (t % RING) * BUFB;
      S[0] = S[1] = dP[0] = dP[1] = (f32x16){0};
      mfma_stream<4 * KS, MASK && D == 128 ? 2 : 4, 1>(  // (mask, d = 128: shorter operand prefetch, the registers go to M)
          [&](int i) {
            const int ks = i >> 2, kt = (i >> 1) & 1;
            return lds_b128(smem, (zk ^ (32 * ks)) + 32 * kt * ROWB + (i & 1) * TILEB);
          },
          [&](int i, bf16x8 x) {
            const int ks = i >> 2, kt = (i >> 1) & 1;
            // (NEGD: the dP products start from -D_i, so that dP - D comes out of the MFMAs)
            if (i & 1) dP[kt] = mfma32<F16>(x, dOf[ks], NEGD && ks == 0 ? negD : dP[kt]);
            else S[kt] = mfma32<F16>(x, Qf[ks], S[kt]);
          });
    }
    if (t > tb && wave_sees(blk(t - 1))) {
      // ---- dQ_i^T += K_{j-1}^T dS^T (line 15), j - 1 the block before this one in the walk
      const int kb = ((t - 1) % RING) * BUFB;
      const int zc0 = zcol[0] + kb, zc1 = zcol[1] + kb;
      mfma_stream<4 * DT, MASK && D == 128 ? 2 : 3, 2>(
          [&](int i) {
            const int dt = i >> 2, ro = (16 * (i & 3)) * ROWB;
            return lds_tr_pair(smem, (zc0 ^ (64 * dt)) + ro, (zc1 ^ (64 * dt)) + ro);
          },
          [&](int i, bf16x8 x) { dQt[i >> 2] = mfma32<F16>(x, dSf[(i >> 1) & 1][i & 1], dQt[i >> 2]); });
    }
    __builtin_amdgcn_s_setprio(0);
  };

  const uint32_t drop_lane = DROPOUT ? (uint32_t)hh * kDropCol + (uint32_t)row * kDropRow +
                                           (p.drop_seed ^ (uint32_t)(s * p.Hq + h) * kDropHead)
                                     : 0u;
  // ================= vector phase j: P = exp(S - L) (line 11), dS = P o (dP - D) (line 14) =================
  auto vector_phase = [&](int t) {
    const int j = blk(t);
    if (t >= tend || !wave_sees(j)) return;
    const int col0 = j * BC;
    const bool need_mask = (CAUSAL && col0 + BC - 1 > wrow0 + off) || (col0 + BC > nk) ||
                           (LOCAL && ((wr >= 0 && col0 + BC - 1 > wrow0 + off + wr) || (wl >= 0 && col0 < wrow_last - wl)));
    int zm = lq * (2 * BC) + ((lq & 7) << 4) + 8 * hh;  // mask: chunk k of this lane's row at zm ^ 16 k
    if constexpr (MASK) {
      wait_vmem_upto<TPW>();  // this piece of M is older than this phase's tile copies
      asm volatile("" : "+v"(zm));  // (recomputed every block instead of held in registers)
    }
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      if constexpr (MASK) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {  // registers 4 q4 .. 4 q4 + 3: keys col0 + 32 kt + 8 q4 + 4 hh + 0..3
          const u32x2 mv = *(const u32x2*)(mbuf + (zm ^ (16 * (4 * kt + q4))));
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float mf = widen_half<F16>(mv[u >> 1], u & 1);
            S[kt][4 * q4 + u] = fast_exp2(__builtin_fmaf(S[kt][4 * q4 + u], c2, __builtin_fmaf(mf, kLog2e, -Lq)));
          }
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) S[kt][r] = fast_exp2(__builtin_fmaf(S[kt][r], c2, -Lq));
      }
      if (need_mask) {  // tiles on the diagonal or at the end of the sequence only
        asm volatile("; keep this a branch: the mask costs three instructions per element" ::);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = col0 + 32 * kt + acc_row(r, hh);
          if (c > lim_row || (LOCAL && c < lo_row)) S[kt][r] = 0.f;
        }
      }
      if constexpr (DROPOUT) {  // dP = keep o (dO V^T) / (1 - p)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {  // registers 4 q4 .. 4 q4 + 3: keys col0 + 32 kt + 8 q4 + 4 hh + 0..3
          const uint32_t x = drop_mix(drop_lane + (uint32_t)(col0 / 4 + 8 * kt + 2 * q4) * kDropCol);
#pragma unroll
          for (int u = 0; u < 4; ++u)
            dP[kt][4 * q4 + u] = ((x >> (8 * u)) & 255u) >= p.drop_thr ? dP[kt][4 * q4 + u] * p.drop_rp : 0.f;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) dP[kt][r] = NEGD ? S[kt][r] * dP[kt][r] : S[kt][r] * (dP[kt][r] - Dq);
      if constexpr (MASK) {
        // dM = dS (the mask enters the scores unscaled): this lane's four groups of four neighbouring
        // keys of its row, 8 bytes each; removed entries have P = 0 and store zeros. Groups that start
        // past the last key are left out (a group may reach up to three columns into the row's padding).
        if (a.dM && row < n) {
          long o = (long)row * a.dm_rs + col0 + 32 * kt + 4 * hh;
          asm volatile("" : "+v"(o));  // (recomputed for every block instead of held in registers)
          __bf16* dst = a.dM + s * a.dm_bs + (long)h * a.dm_hs + o;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            u32x2 x;
            x[0] = pack2<F16>(dP[kt][4 * q4], dP[kt][4 * q4 + 1]);
            x[1] = pack2<F16>(dP[kt][4 * q4 + 2], dP[kt][4 * q4 + 3]);
            if (col0 + 32 * kt + 8 * q4 + 4 * hh < nk) *(u32x2*)(dst + 8 * q4) = x;
          }
        }
      }
      dSf[kt][0] = pack8<F16>(dP[kt], 0);
      dSf[kt][1] = pack8<F16>(dP[kt], 1);
    }
  };

  // phases: see the forward kernel (j counts positions of the walk; one barrier per block, the one
  // between a group's matrix and vector phase is left out as in the forward kernel's one-workgroup form)
  if (grp == 0) {
    for (int j = tb; j <= tend; ++j) {
      matrix_phase(j);
      issue_tile(j + 2);
      vector_phase(j);
      issue_mask(j + 1);
      wait_vmem_upto<TPW + MPW>();
      lds_barrier();
    }
  } else {
    issue_tile(tb + 2);
    for (int j = tb; j <= tend; ++j) {
      matrix_phase(j);
      wait_vmem_upto<TPW + MPW>();
      lds_barrier();
      if (j < tend) {
        issue_tile(j + 3);
        vector_phase(j);
        issue_mask(j + 1);
      }
    }
  }

  {
    // dQ_i through the one ring slot that is neither in use nor the target of a copy issued
    // past the last block, as whole rows (see store_rows_via_lds)
    static_assert(RING == 4 && BUFB / 8 == 32 * D, "the staging area of a wavefront is an eighth of a ring slot");
    char* stg = smem + ((tend + 3) % RING) * BUFB + w * (BUFB / 8);
    __bf16* op = a.dQ + ((si.tok0 + wrow0) * p.Hq + h) * dh;
    const long ostride = (long)p.Hq * dh;
    int ln = lane;  // recomputed here: nothing of the staging addresses is to live across the main loop
    asm volatile("" : "+v"(ln));
    if constexpr (DT % 2 == 0) {
#pragma unroll
      for (int half = 0; half < 2; ++half)
        store_rows_via_lds<DT / 2, F16>(stg, &dQt[half * (DT / 2)], p.scale, op + half * (DH / 2), ostride, n - wrow0,
                                        dh - half * (DH / 2), ln);
    } else {  // (an odd number of 32-column tiles: one at a time)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        store_rows_via_lds<1, F16>(stg, &dQt[dt], p.scale, op + 32 * dt, ostride, n - wrow0, dh - 32 * dt, ln);
    }
  }
}

template <int D, bool F16>
static hipError_t launch_bwd_d(const BwdArgs& a, int causal, int stages, hipStream_t st) {
  const long nrows = (long)a.p.total_tokens * a.p.Hq;
  constexpr int RPB = 256 / (D / 8);
  constexpr int DN = D == 128 ? 96 : 32;  // the narrower product width of this tile width (padded head dimensions)
  hipError_t e = hipSuccess;
  // The whole backward on the plain paths (no dropout, mask, window or pattern): two launches. The
  // dQ kernel goes first and computes D on the way, the dK/dV kernel follows and reads it.
  const bool plain = !a.p.mask && !a.p.drop_thr && !a.p.bmask && a.p.win_left < 0 && a.p.win_right < 0;
  if (stages == 7 && plain) {
    dim3 qgrid(grid_size((a.p.N + 255) / 256, a.p.Hq * a.p.nseq));
    if (a.p.d != D && a.p.d <= DN) {
      if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16, false, true, false, false, true, DN>), qgrid, dim3(512), 0, st, a);
      else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, false, true, false, false, true, DN>), qgrid, dim3(512), 0, st, a);
    } else if (a.p.d != D) {
      if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16, false, true, false, false, true>), qgrid, dim3(512), 0, st, a);
      else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, false, true, false, false, true>), qgrid, dim3(512), 0, st, a);
    } else {
      if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16, false, false, false, false, true>), qgrid, dim3(512), 0, st, a);
      else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, false, false, false, false, true>), qgrid, dim3(512), 0, st, a);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    stages = 2;  // what remains: the dK/dV kernel
  } else if (stages == 7 && a.p.d == D) {  // sliding window or block-sparse pattern, mask, dropout: the same two launches
    dim3 qgrid(grid_size((a.p.N + 255) / 256, a.p.Hq * a.p.nseq));
    if (a.p.mask) {
      if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16, false, false, true, false, true>), qgrid, dim3(512), 0, st, a);
      else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, false, false, true, false, true>), qgrid, dim3(512), 0, st, a);
    } else if (a.p.drop_thr) {
      if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16, true, false, false, false, true>), qgrid, dim3(512), 0, st, a);
      else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, true, false, false, false, true>), qgrid, dim3(512), 0, st, a);
    } else {
      hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, false, false, false, true, true>), qgrid, dim3(512), 0, st, a);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    stages = 2;
  }
  if (stages & 1) {
    hipLaunchKernelGGL((bwd_prep_kernel<D, F16>), dim3((unsigned)((nrows + RPB - 1) / RPB)), dim3(256), 0, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (stages & 2) {
    // keys per workgroup differ between the instantiations
    const bool special = a.p.mask || a.p.drop_thr;
    const int bck = special ? dkdv_block_keys(D, true, true) : dkdv_block_keys(D, false, false);
    dim3 grid(grid_size((a.p.Nk + bck - 1) / bck, a.p.Hkv * a.p.nseq));
    bool done = false;
    {
      if (a.p.win_left >= 0 || a.p.win_right >= 0 || a.p.bmask) {  // sliding window, block-sparse pattern
        hipLaunchKernelGGL((bwd_dkdv_kernel<D, false, F16, false, false, false, true>), grid, dim3(512), 0, st, a);
        done = true;
      } else
      if (a.p.mask) {
        if (causal) hipLaunchKernelGGL((bwd_dkdv_kernel<D, true, F16, false, false, true>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((bwd_dkdv_kernel<D, false, F16, false, false, true>), grid, dim3(512), 0, st, a);
        done = true;
      }
    }
    if (done) {
    } else if (a.p.d != D) {  // padded head dimension (the entry points keep dropout away from it)
      if (a.p.d <= DN) {
        if (causal) hipLaunchKernelGGL((bwd_dkdv_kernel<D, true, F16, false, true, false, false, DN>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((bwd_dkdv_kernel<D, false, F16, false, true, false, false, DN>), grid, dim3(512), 0, st, a);
      } else {
        if (causal) hipLaunchKernelGGL((bwd_dkdv_kernel<D, true, F16, false, true>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((bwd_dkdv_kernel<D, false, F16, false, true>), grid, dim3(512), 0, st, a);
      }
      done = true;
    }
    {
      if (!done && a.p.drop_thr) {
        if (causal) hipLaunchKernelGGL((bwd_dkdv_kernel<D, true, F16, true>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((bwd_dkdv_kernel<D, false, F16, true>), grid, dim3(512), 0, st, a);
        done = true;
      }
    }
    if (done) {
    } else if (causal) hipLaunchKernelGGL((bwd_dkdv_kernel<D, true, F16>), grid, dim3(512), 0, st, a);
    else hipLaunchKernelGGL((bwd_dkdv_kernel<D, false, F16>), grid, dim3(512), 0, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (stages & 4) {
    dim3 grid(grid_size((a.p.N + 255) / 256, a.p.Hq * a.p.nseq));
    bool done = false;
    {
      if (a.p.win_left >= 0 || a.p.win_right >= 0 || a.p.bmask) {  // sliding window, block-sparse pattern
        hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, false, false, false, true>), grid, dim3(512), 0, st, a);
        done = true;
      } else
      if (a.p.mask) {
        if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16, false, false, true>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, false, false, true>), grid, dim3(512), 0, st, a);
        done = true;
      }
    }
    if (done) {
    } else if (a.p.d != D) {
      if (a.p.d <= DN) {
        if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16, false, true, false, false, false, DN>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, false, true, false, false, false, DN>), grid, dim3(512), 0, st, a);
      } else {
        if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16, false, true>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, false, true>), grid, dim3(512), 0, st, a);
      }
      done = true;
    }
    {
      if (!done && a.p.drop_thr) {
        if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16, true>), grid, dim3(512), 0, st, a);
        else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16, true>), grid, dim3(512), 0, st, a);
        done = true;
      }
    }
    if (done) {
    } else if (causal) hipLaunchKernelGGL((bwd_dq_kernel<D, true, F16>), grid, dim3(512), 0, st, a);
    else hipLaunchKernelGGL((bwd_dq_kernel<D, false, F16>), grid, dim3(512), 0, st, a);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_bwd(const BwdArgs& a, int d, int causal, int stages, hipStream_t st) {
  if (stages & 4)
    if (hipError_t e = launch_keyless_rows(a.p, a.dQ, nullptr, st)) return e;
  if (d == 256) {  // the D pre-pass is the generic one, the two kernels live in fa_d256.hip
    if (stages & 1) {
      const long nrows = (long)a.p.total_tokens * a.p.Hq;
      constexpr int RPB = 256 / (256 / 8);
      if (a.p.f16) hipLaunchKernelGGL((bwd_prep_kernel<256, true>), dim3((unsigned)((nrows + RPB - 1) / RPB)), dim3(256), 0, st, a);
      else hipLaunchKernelGGL((bwd_prep_kernel<256, false>), dim3((unsigned)((nrows + RPB - 1) / RPB)), dim3(256), 0, st, a);
      if (hipError_t e = hipGetLastError()) return e;
    }
    return launch_bwd256(a, causal, stages, st);
  }
  if (a.p.f16) return d <= 64 ? launch_bwd_d<64, true>(a, causal, stages, st) : launch_bwd_d<128, true>(a, causal, stages, st);
  return d <= 64 ? launch_bwd_d<64, false>(a, causal, stages, st) : launch_bwd_d<128, false>(a, causal, stages, st);
}

}  // namespace fa
