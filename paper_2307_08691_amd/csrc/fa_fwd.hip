// Forward pass of exact attention for gfx950 (Algorithm 1 of the paper).
//
// One workgroup (8 wavefronts) owns one block of BR = 256 query rows of one
// (sequence, query head) and walks the key/value sequence in blocks of BC = 64
// (the inner loop over column blocks j; the outer loop over row blocks i is the
// grid, section 3.2 "Forward pass"). Each wavefront owns 32 whole query rows, so
// no reduction between wavefronts is ever needed (section 3.3).
//
// The scores are computed TRANSPOSED, S^T = K_j Q_i^T, with 32x32x16 bf16 MFMAs:
// a lane then holds 16 keys of ONE query per 32x32 tile, the row maximum and row
// sum are in-lane reductions plus a single exchange with lane ^ 32, and the
// exponentiated tile, rounded to bf16, is already in the operand layout of the
// second product O^T += V_j^T P^T. V_j^T operands come from transposing LDS reads
// of the row-major V tile, so nothing is ever transposed in memory.
//
// Phases. Two wavefronts share a SIMD, and left alone they run the same instruction stream
// in step: both want the matrix pipe at the same time and both leave it idle during their
// softmax. The loop is therefore cut into phases separated by workgroup barriers: a matrix
// phase (S^T for block j and the O^T update with block j-1) and a vector phase (the online
// softmax of block j). Wavefronts 0-3 and 4-7, which share the four SIMDs pairwise, run the
// same program one phase apart, so at any time one wavefront of every SIMD is in its matrix
// phase (at raised priority) and the other in its vector phase. The alternative without
// phases - each wavefront slicing the softmax of block j between the MFMAs of blocks j-1
// and j+1, scores double buffered, one barrier per block - measured 1.24 ms against 1.05 ms
// for this form (d = 128, N = 8192, 32 heads, no mask).
//
// K_j and V_j travel HBM -> LDS directly (no registers), two blocks ahead, into a
// ring of four swizzled (unpadded) buffers shared by all eight wavefronts.
//
// Two kernels: fwd_kernel (every option: split keys, half precision, dropout, padded head
// dimension, elementwise mask) and fwd_chain_kernel (d = 128, short dense sequences: several
// row blocks per workgroup, each one's start-up hidden behind the previous one's last blocks).
#include <type_traits>

#include "fa_common.h"
#include "fa_kernels.h"
#include "fa_lds.h"

namespace fa {

// How many MFMAs ahead the LDS operands of the two products are requested.
constexpr int kFwdAheadQK = 4, kFwdAheadPV = 3;
// Wave priority of a matrix phase: the MFMA stream must not wait behind the other group's
// vector work (measured: 3-5% slower at d = 128 without it).
#define FA_FWD_MATRIX_PRIO 2
// The reference of the running softmax is only advanced (and O, l rescaled) when a lane's share
// of a block's row sum exceeds 2^kFwdLazyLog2 (instantiations without the fast path: when some
// row's maximum outgrew the reference by that factor); until then exponentials are taken against
// the older reference and may reach 2^kFwdLazyLog2. Half precision operands end at 65504 = 2^16;
// bfloat16 has float32's range, and the wider margin saves most of the remaining advances when the
// scores spread widely (3x the usual range: the row maximum grows by some 20 bits over 16k keys).
constexpr int kFwdLazyLog2Half = 8, kFwdLazyLog2Bf16 = 20;
// d = 128: workgroups that take several items in a row and overlap an item's start-up with the
// end of the one before (fwd_chain_kernel), for sequences of at most kFwdChainMaxN keys
constexpr int kFwdChainMaxN = 1024;

// At d = 64 the kernel needs 64 KiB of LDS, so two workgroups fit on a compute unit if their
// 16 wavefronts do, i.e. with at most 128 registers each. Two resident workgroups overlap one's
// start-up (Q and the first tiles: one memory latency) and epilogue with the other's loop,
// which a single workgroup per compute unit cannot: 10% faster at N = 8192, 27% at N = 512.
// The price is the shortest operand prefetch (one MFMA ahead). Not for dropout (more
// registers) or the elementwise mask (more LDS).
constexpr bool fwd_two_per_cu(int D, bool dropout, bool mask) { return D == 64 && !dropout && !mask; }

__device__ __forceinline__ float max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// SPLIT (forward only, few query rows against many keys): the workgroups of one (sequence,
// key/value head) also split the KEY sequence, each writing a normalised partial O and its
// logsumexp in float32; fwd_merge_kernel combines them with the identity the paper uses
// between blocks, O = sum_k e^{L_k - L} O_k, L = logsumexp_k L_k (section 3.1.1). The G query
// heads that share the key/value head are packed into the row block (row = query * G + head),
// so K and V are read once for all of them.
//
// PAD: the head dimension in memory, p.d, is smaller than the tile width D. Rows are padded
// with zeros on chip (registers for Q, never-written LDS chunks for K and V), which changes
// no product, and only the first p.d columns of O are stored.
//
// MASK: a tensor M is added to the scaled scores before the softmax (section 2.2, footnote).
// Each wavefront copies its own 32 x 64 piece of M for the next block HBM -> LDS at the end
// of its vector phase (a private 4 KiB buffer, 16-byte chunks XOR-ed with the row so that the
// 8-byte reads of 32 rows spread over all banks) and adds it, times log2(e), to the scores in
// the exponent's base at the start of the next one. Entries of -inf remove a score; a row may
// be left without any, so the running maximum can stay -inf (guards as for SPLIT) and such a
// row ends with O = 0, L = -inf.
//
// LOCAL: a sliding window (section 5 names local attention as a pattern to combine with; the
// block skipping of section 3.1.1 carries over): key c is visible to the query at position q
// iff q - win_left <= c <= q + win_right. The workgroup walks only the column blocks its rows
// can see, a wavefront sits out the blocks none of its 32 rows can see, and the element mask
// is applied on the blocks that straddle an edge of the band. A row's first visible key may
// lie in a later block than its wavefront's first one, so the guards for "no key seen yet"
// of the split-key kernel apply. Instantiated with CAUSAL = false (win_right = 0 is the rule).
//
// DH (PAD only): the head dimension rounded up to a multiple of 32. The tiles in LDS keep the
// width D (row pitch, swizzle and copies are those of the full tile), but the products only run
// over the first DH columns: D = 128 with DH = 96 does three quarters of the matrix work of the
// full width, D = 64 with DH = 32 half.
template <int D, bool CAUSAL, bool SPLIT, bool F16, bool DROPOUT = false, bool PAD = false, bool MASK = false,
          bool LOCAL = false, int DH = D>
__global__ __launch_bounds__(512)
    __attribute__((amdgpu_waves_per_eu(fwd_two_per_cu(D, DROPOUT, MASK || LOCAL) ? 4 : 2, fwd_two_per_cu(D, DROPOUT, MASK || LOCAL) ? 4 : 2))) void
    fwd_kernel(FwdArgs a) {
  constexpr bool TWO = fwd_two_per_cu(D, DROPOUT, MASK || LOCAL);
  static_assert(!LOCAL || (!CAUSAL && !SPLIT && !DROPOUT && !PAD && !MASK), "the window variant is built for the plain kernel");
  constexpr int AHEAD_QK = TWO ? 1 : kFwdAheadQK, AHEAD_PV = TWO ? 1 : kFwdAheadPV;
  static_assert(!MASK || (!SPLIT && !DROPOUT && !PAD), "the mask variant is built for the plain kernel");
  constexpr int BR = 256, BC = 64, RING = 4;
  static_assert(DH == D || (PAD && DH % 32 == 0 && DH < D), "a narrower product width is for padded head dimensions");
  constexpr int KS = DH / 16;  // contraction steps of the first product
  constexpr int DT = DH / 32;  // 32-row tiles of O^T
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = BC * ROWB, BUFB = 2 * TILEB;  // one buffer = K_j | V_j

  constexpr int MASKB = 32 * BC * 2;             // one wavefront's piece of M for one block
  constexpr int MPW = MASK ? MASKB / 1024 : 0;  // copies per wavefront per block

  // (LOCAL: behind the ring, one bitmap of kPatternWords 64-bit words per wavefront: which key blocks
  // the block-sparse pattern leaves to its rows; behind them the list of the key blocks that it
  // leaves to any row of the workgroup, two bytes each)
  constexpr int BITSB = 8 * 8 * kPatternWords, LISTB = 2 * 64 * kPatternWords;
  __shared__ __attribute__((aligned(1024))) char smem[RING * BUFB + (MASK ? 8 * MASKB : 0) + (LOCAL ? BITSB + LISTB : 0)];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = w >> 2;  // 0: matrix phase on even phases, 1: on odd phases
  const int lq = lane & 31, hh = lane >> 5;
  const int nsplit = SPLIT ? a.nsplit : 1;
  const int nblk = ((SPLIT ? p.N * p.G : p.N) + BR - 1) / BR;
  const BlockCoord bc = block_coord<CAUSAL && !SPLIT>(nblk * nsplit, SPLIT ? p.Hkv : p.Hq, p.nseq, SPLIT ? 1 : p.G);
  if (!bc.valid) return;
  const int split = SPLIT ? bc.blk % nsplit : 0;
  const int rowblk = SPLIT ? bc.blk / nsplit : nblk - 1 - bc.blk;  // not split: longest causal rows first
  const int s = bc.seq;
  const SeqInfo si = seq_info(p, s);
  int nk_ = si.nk;
  if (SPLIT && a.seqlens_k) {  // a key/value cache filled up to a length of its own per sequence
    const int len = a.seqlens_k[s];
    nk_ = len < 0 ? 0 : (len < p.Nk ? len : p.Nk);
  }
  const int n = si.n, nk = nk_;  // query rows, key rows
  const int off = nk - n;          // position of query 0 among the keys (causal alignment)
  const int nrows = SPLIT ? n * p.G : n;  // rows of the (packed) row dimension
  const int i0 = rowblk * BR;
  if (i0 >= nrows || nk == 0) return;  // (a sequence without keys: see keyless_rows_kernel, fwd_merge_kernel)
  const int g = SPLIT ? bc.head : bc.head / p.G;
  const int dh = PAD ? p.d : D;  // row length in memory
  const long kstride = (long)p.Hkv * dh;
  const __bf16* Kb = a.K + (si.tok0k * p.Hkv + g) * dh;
  const __bf16* Vb = a.V + (si.tok0k * p.Hkv + g) * dh;
  if (PAD) lds_zero<512>(smem, RING * BUFB);

  // ---- Q_i operands: registers for the whole kernel (Algorithm 1, line 4)
  // row: this lane's query (index into the sequence), h: its head. Packed rows interleave the
  // heads of the group, so both are per lane there.
  const int prow0 = i0 + 32 * w;  // first (packed) row of this wavefront
  const int prow = prow0 + lq;
  const bool row_ok = prow < nrows;
  const int prowc = row_ok ? prow : nrows - 1;  // rows past the end compute on a copy and are never stored
  const int row = SPLIT ? prowc / p.G : prow;
  const int rowc = SPLIT ? row : prowc;
  const int h = SPLIT ? g * p.G + prowc % p.G : bc.head;
  const int prow_last = prow0 + 31 < nrows ? prow0 + 31 : nrows - 1;
  const int wrow0 = SPLIT ? prow0 / p.G : prow0;             // first and last query of this wavefront
  const int wq_last = SPLIT ? prow_last / p.G : prow0 + 31;
  const bool wave_on = !SPLIT || prow0 < nrows;  // a wavefront without rows only helps with the copies
  bf16x8 Qf[KS];
  {
    const __bf16* qp = a.Q + ((si.tok0 + rowc) * p.Hq + h) * dh + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Qf[ks] = (bf16x8){0};
      if (!PAD || 16 * ks + 8 * hh < dh) Qf[ks] = *(const bf16x8*)(qp + 16 * ks);
    }
  }

  // ---- on-chip state (Algorithm 1, line 5)
  f32x16 O[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x16){0};
  float m = -INFINITY;  // running row maximum, raw score units (mask: scaled scores, M included)
  float l = 0.f;        // this lane's share of the row sum (the two lane halves are added at the end)

  // column blocks the workgroup visits: all of them, or (causal) those not entirely above the diagonal
  // (split: this workgroup's share jb .. of them)
  const int ncol_all = (nk + BC - 1) / BC;
  const int per_split = (ncol_all + nsplit - 1) / nsplit;
  int jb = split * per_split;
  int ncol = jb + per_split < ncol_all ? jb + per_split : ncol_all;
  const int wl = LOCAL ? p.win_left : -1, wr = LOCAL ? p.win_right : -1;  // window bounds (negative: none)
  if (CAUSAL || LOCAL) {
    const int last_prow = (i0 + BR < nrows ? i0 + BR : nrows) - 1;
    const int last_pos = (SPLIT ? last_prow / p.G : last_prow) + off;
    if (CAUSAL || wr >= 0) {
      const int c = (last_pos + (LOCAL ? wr : 0)) / BC + 1;
      ncol = c < ncol ? c : ncol;
    }
    if (LOCAL && wl >= 0 && i0 + off > wl) jb = (i0 + off - wl) / BC;  // the first block the first row sees
  }
  if (SPLIT && jb >= ncol) {  // this share holds no key that the workgroup's rows see: L = -inf says so to the merge
    if (row_ok && hh == 0)
      a.Lpart[(long)split * p.total_tokens * p.Hq + s * p.lse_seq_stride + h * p.lse_head_stride + row] = -INFINITY;
    return;
  }
  if (ncol < jb) ncol = jb;  // nothing visible: the loops below still run once

  // Block-sparse pattern: the wavefront's 32 rows lie in one row block of the pattern (blocks are
  // at least 64 rows and the wavefront starts at a multiple of 32), so whether it has anything to
  // do in key block j is one bit, gathered here for every j (one byte per lane and ballot) into
  // the wavefront's bitmap. It is read back a word at a time.
  // The workgroup then walks only the blocks that some wavefront of it has a bit for: every
  // wavefront compacts the union of the eight bitmaps (inside jb .. ncol) into the same list, so
  // neither copies nor phases are spent on a block that the pattern removes from all 256 rows.
  const unsigned long long* pattern_bits = (const unsigned long long*)(smem + RING * BUFB) + w * kPatternWords;
  const unsigned short* visit = (const unsigned short*)(smem + RING * BUFB + BITSB);
  const bool sparse = LOCAL && p.bmask != nullptr;
  int tb = jb, tend = ncol;  // positions of the walk; position t stands for block t unless the pattern thins the walk
  bool listed = false;       // the walk follows the list
  if (LOCAL && sparse) {
    const int r0 = prow0 < n ? prow0 : n - 1;
    const uint8_t* bm_row = p.bmask + s * p.bmask_bs + bc.head * p.bmask_hs + (long)(r0 >> p.bmask_log2) * p.bmask_cols;
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

  // Tile loads. Issuing a tile's copies stalls the issuing wavefronts for a few hundred
  // cycles (the memory pipeline takes 16 bytes x 64 lanes at a time), so a wavefront only
  // issues copies at the start of its VECTOR phase, while the other group keeps the MFMA pipe
  // busy: group 1 brings in the K tiles, group 0 the V tiles, each two blocks ahead. Every
  // wavefront issues exactly TPW copies per own vector phase, also past the last block (rows
  // are clamped, the data is never read), so the waits below can count instructions.
  TileLoader<D, BC, 4, PAD> loader;
  loader.init(kstride, w & 3, lane, dh / 8);
  constexpr int TPW = TileLoader<D, BC, 4, PAD>::PER;  // copies per wavefront per tile
  auto issue_tile = [&](int t) {  // the block at position t of the walk; group 0: its V_j, group 1: its K_j
    char* dst = smem + (t % RING) * BUFB + (grp == 0 ? TILEB : 0);
    if (SPLIT && a.block_table) {
      // paged cache: a block of 64 keys lies inside one page (pages are multiples of 64 rows);
      // copies past the last block fetch the last block again (never read)
      const int jc = t < ncol_all ? t : ncol_all - 1;
      const int key0 = jc * BC, in_page = key0 & ((1 << a.page_log2) - 1);
      const int pg = __builtin_amdgcn_readfirstlane(a.block_table[(long)s * a.table_stride + (key0 >> a.page_log2)]);
      const __bf16* base = (grp == 0 ? a.V : a.K) + (((long)pg << a.page_log2) * p.Hkv + g) * dh;
      const int last = nk - 1 - (key0 - in_page);  // the sequence's last key, counted from the page's first row
      loader.load(dst, base, kstride, in_page, last < (1 << a.page_log2) - 1 ? last : (1 << a.page_log2) - 1, w & 3, lane);
      return;
    }
    loader.load(dst, grp == 0 ? Vb : Kb, kstride, blk(t) * BC, nk - 1, w & 3, lane);
  };
  // MASK: this wavefront's rows of M, columns of block j (rows and columns clamped into the
  // tensor: what lies past the end is never used). Issued unconditionally, once per vector
  // phase, like the tile copies, so that the waits can count instructions.
  char* mbuf = smem + RING * BUFB + w * MASKB;
  const __bf16* Mb = MASK ? p.mask + s * p.mask_bs + h * p.mask_hs : nullptr;
  const int nk8 = (nk + 7) & ~7;
  auto issue_mask = [&](int j) {
    if constexpr (MASK) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the reads of the previous piece have returned
      int ln = lane;  // hidden from the optimiser: otherwise it keeps all these addresses in registers across the loop
      asm volatile("" : "+v"(ln));
#pragma unroll
      for (int u = 0; u < MPW; ++u) {
        const int r = 8 * u + (ln >> 3);
        const int qr = prow0 + r < n ? prow0 + r : n - 1;
        const int c = (ln & 7) ^ (r & 7);
        int col = j * BC + 8 * c;
        col = col < nk8 ? col : 0;
        dma16(Mb + (long)qr * p.mask_rs + col, mbuf + u * 1024);
      }
    }
  };
  {  // the first two blocks: both tiles, split over the two groups as above
    issue_tile(tb);
    issue_tile(tb + 1);
    issue_mask(jb);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) touch(Qf[ks]);
    wait_vmem();
    lds_barrier();
  }

  // lane constants of the LDS addressing (see fa_lds.h)
  const int zrow = lq * ROWB + 16 * (hh ^ swz<ROWB>(lq));
  const int p16 = lane & 15, g16 = (lane >> 4) & 1;
  int zcol[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
    zcol[u] = swz_off<ROWB>(4 * hh + (p16 >> 2) + 8 * u, 2 * g16 + ((p16 & 3) >> 1)) + 8 * (p16 & 1);

  const float c2 = p.scale_log2e;
  constexpr bool GUARD = SPLIT || MASK || LOCAL;  // a row may have seen no key yet
  // MASK: the scores are scaled when M is added (one FMA); from there on the softmax works on
  // scaled scores and the factor that remains is the change of base
  const float cs = MASK ? kLog2e : c2;
  const int wrow_last = wq_last + off;  // position of the wavefront's last query among the keys
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

  f32x16 S[2];
  bf16x8 Pf[2][2];
  // dropout: this lane's part of the hash input (its query row, its lane half, its head)
  const uint32_t drop_lane = DROPOUT ? (uint32_t)hh * kDropCol + (uint32_t)row * kDropRow +
                                           (p.drop_seed ^ (uint32_t)(s * p.Hq + h) * kDropHead)
                                     : 0u;

  // ================= matrix phase j: S^T of block j, O^T update with block j - 1 =================
  auto matrix_phase = [&](int t) {
    __builtin_amdgcn_s_setprio(FA_FWD_MATRIX_PRIO);  // the MFMA stream must not wait behind the other group's VALU work
    if (wave_on && t < tend && wave_sees(blk(t))) {
      // ---- S^T = K_j Q_i^T (Algorithm 1, line 8)
      const int zk = zrow + (t % RING) * BUFB;
      S[0] = S[1] = (f32x16){0};
      mfma_stream<2 * KS, AHEAD_QK, 1>(
          [&](int i) { return lds_b128(smem, (zk ^ (32 * (i >> 1))) + (i & 1) * 32 * ROWB); },
          [&](int i, bf16x8 x) { S[i & 1] = mfma32<F16>(x, Qf[i >> 1], S[i & 1]); });
    }
    if (wave_on && t > tb && wave_sees(blk(t - 1))) {
      // ---- O^T += V_{j-1}^T P^T (Algorithm 1, line 10), j - 1 the block before this one in the walk
      const int vb = ((t - 1) % RING) * BUFB + TILEB;
      const int zv0 = zcol[0] + vb, zv1 = zcol[1] + vb;
      mfma_stream<4 * DT, AHEAD_PV, 2>(
          [&](int i) {
            const int dt = i >> 2, ro = (16 * (i & 3)) * ROWB;
            return lds_tr_pair(smem, (zv0 ^ (64 * dt)) + ro, (zv1 ^ (64 * dt)) + ro);
          },
          [&](int i, bf16x8 x) { O[i >> 2] = mfma32<F16>(x, Pf[(i >> 1) & 1][i & 1], O[i >> 2]); });
    }
    __builtin_amdgcn_s_setprio(0);
  };

  // ================= vector phase j: online softmax of block j (Algorithm 1, line 9) =================
  auto vector_phase = [&](int t) {
    const int j = blk(t);
    if (!wave_on || t >= tend || !wave_sees(j)) return;
    const int col0 = j * BC;
    if constexpr (MASK) {
      wait_vmem_upto<TPW>();  // the copies of this piece of M are older than this phase's tile copies
      int zm = lq * (2 * BC) + ((lq & 7) << 4) + 8 * hh;  // chunk k of this lane's row: zm ^ 16 k
      asm volatile("" : "+v"(zm));                        // (recomputed every block instead of held in registers)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {  // registers 4 q4 .. 4 q4 + 3: keys col0 + 32 kt + 8 q4 + 4 hh + 0..3
          const u32x2 mv = *(const u32x2*)(mbuf + (zm ^ (16 * (4 * kt + q4))));
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float mf = widen_half<F16>(mv[u >> 1], u & 1);
            S[kt][4 * q4 + u] = __builtin_fmaf(S[kt][4 * q4 + u], p.scale, mf);
          }
        }
    }
    // ---- mask: causal entries above the diagonal and columns past the end
    const bool need_mask = (CAUSAL && col0 + BC - 1 > wrow0 + off) || (col0 + BC > nk) ||
                           (LOCAL && ((wr >= 0 && col0 + BC - 1 > wrow0 + off + wr) || (wl >= 0 && col0 < wrow_last - wl)));
    if (need_mask) {
      asm volatile("; keep this a branch: the mask costs two instructions per element" ::);
      const int lim = lim_row - col0 - 4 * hh;  // last visible column, relative to this lane's first
      const int lo = lo_row - col0 - 4 * hh;    // (window) first visible column, likewise
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int x = 32 * kt + acc_row(r, 0);
          S[kt][r] = x > lim || (LOCAL && x < lo) ? -INFINITY : S[kt][r];
        }
    }
    // The exponentials of the block against reference `ref` (already in the exponent's base),
    // rounded into the operand registers of the second product; the row sum is taken from the
    // float32 exponentials, not from their bf16 roundings: rows that see only a few keys would
    // otherwise miss the 1e-3 bound on L. On the fast path S itself stays intact.
    constexpr bool FAST = !GUARD && !(PAD && TWO);  // (see below)
    float rs0, rs1;
    auto exponentials = [&](float ref) {
      rs0 = rs1 = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        f32x16 Etmp;
        f32x16& E = FAST ? Etmp : S[kt];  // without the fast path nobody needs S again: in place
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          E[r] = fast_exp2(__builtin_fmaf(S[kt][r], cs, -ref));
          E[r + 1] = fast_exp2(__builtin_fmaf(S[kt][r + 1], cs, -ref));
          rs0 += E[r];
          rs1 += E[r + 1];
        }
        if constexpr (DROPOUT) {  // the row sum above is that of the undropped block; O only sees the kept entries
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {  // registers 4 q4 .. 4 q4 + 3: keys col0 + 32 kt + 8 q4 + 4 hh + 0..3
            const uint32_t x = drop_mix(drop_lane + (uint32_t)(col0 / 4 + 8 * kt + 2 * q4) * kDropCol);
#pragma unroll
            for (int u = 0; u < 4; ++u) E[4 * q4 + u] = ((x >> (8 * u)) & 255u) >= p.drop_thr ? E[4 * q4 + u] : 0.f;
          }
        }
        Pf[kt][0] = pack8<F16>(E, 0);
        Pf[kt][1] = pack8<F16>(E, 1);
      }
    };
    // The reference m of the running softmax need not be the row maximum: O and l are relative to
    // the same reference whatever it is, and rescaling O (line 10) by exp(m_old - m_new) only
    // matters for the range of the numbers. So the row maximum is NOT computed for every block.
    // The block's exponentials are taken against the reference as it stands; only if some lane's
    // share of a row sum then exceeds 2^kFwdLazyLog2 (which also catches an overflow to inf)
    // is the maximum of the block found, the reference advanced to it, O and l rescaled, and the
    // exponentials taken again. After the first few blocks that is rare: the fast path saves the
    // 16 three-way maxima, the exchange with the partner lane and the comparison per block.
    // The first block of a row (m = -inf) always takes the second path, and so do the
    // instantiations in which a row may still have seen no key (split keys, elementwise mask)
    // and the one that has no registers left to keep S beside the exponentials.
    bool advance = !FAST || t == tb;
    if (!advance) {
      exponentials(m * cs);
      advance = __builtin_amdgcn_ballot_w64(rs0 + rs1 > (float)(1 << (F16 ? kFwdLazyLog2Half : kFwdLazyLog2Bf16))) != 0;
    }
    if (advance) {
      float mx = max3(S[0][0], S[0][1], S[1][0]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = max3(mx, S[0][r], S[0][r + 1]);
      mx = max3(mx, S[1][1], S[1][2]);
      mx = fmaxf(mx, S[1][3]);
#pragma unroll
      for (int r = 4; r < 16; r += 2) mx = max3(mx, S[1][r], S[1][r + 1]);
      mx = max_with_partner32(mx);
      const float m_new = fmaxf(m, mx);
      // column 0 is visible to every row and blocks are walked in ascending order, so m_new is
      // finite from the first block on and exp2(-inf) = 0 covers the start (not so with split
      // keys or a mask: GUARD). Without the fast path the reference is advanced only when some
      // row's maximum outgrew it by a factor 2^kFwdLazyLog2.
      if (FAST || __builtin_amdgcn_ballot_w64((m_new - m) * cs > (float)(F16 ? kFwdLazyLog2Half : kFwdLazyLog2Bf16)) != 0) {
        // (split, mask: a row that has still seen no key has m = m_new = -inf and nothing to rescale)
        const float alpha = GUARD && m_new == -INFINITY ? 1.f : fast_exp2((m - m_new) * cs);
        l *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
        m = m_new;
      }
      // (split, mask: a row may have seen no key yet; its scores are all -inf and must give P = 0)
      exponentials((GUARD && m == -INFINITY ? 0.f : m) * cs);
    }
    l += rs0 + rs1;
  };

  // Global phases phi = 0 .. 2 * ncol + 1, a barrier after each. Group 0 runs matrix phase j at
  // phi = 2j and vector phase j at phi = 2j + 1; group 1 runs one phase later. K_{m+2} is
  // requested (by group 1) at phi = 2m and first read at phi = 2m + 4; V_{m+2} is requested
  // (by group 0) at phi = 2m + 1 and first read at phi = 2m + 6. A group waits, at the end of
  // a later phase of its own, until only its newest tile is still in flight.
  // (j counts positions of the walk: the blocks themselves unless a pattern thins the walk)
  //
  // With one workgroup per compute unit only every second of those barriers is kept (MID false):
  // the one after group 0's vector phase j / group 1's matrix phase j. It alone orders everything
  // that goes through LDS: a tile is requested two barriers before its first reader starts, its
  // copies are waited for right before the barrier in between, and the slot it takes was last read
  // (K_{j-2} in matrix phase j - 2, V_{j-2} in matrix phase j - 1 of both groups) before the barrier
  // that precedes the request. What the barrier in the middle added was that the two wavefronts of a
  // SIMD change phase together; without it a matrix phase that ends early runs into the vector phase
  // at once instead of waiting for the other group (+2% at d = 128; with two workgroups per compute
  // unit, four wavefronts per SIMD, it measured 3% slower and stays).
  constexpr bool MID = TWO;
  if (grp == 0) {
    for (int j = tb; j <= tend; ++j) {
      matrix_phase(j);
      if (MID) lds_barrier();
      issue_tile(j + 2);
      vector_phase(j);
      issue_mask(j + 1);
      wait_vmem_upto<TPW + MPW>();
      lds_barrier();
    }
  } else {
    issue_tile(tb + 2);
    if (MID) lds_barrier();
    for (int j = tb; j <= tend; ++j) {
      matrix_phase(j);
      wait_vmem_upto<TPW + MPW>();
      lds_barrier();
      if (j < tend) {
        issue_tile(j + 3);
        vector_phase(j);
        issue_mask(j + 1);
        if (MID) lds_barrier();
      }
    }
  }

  // ---- epilogue: O = diag(l)^-1 O, L = m + log l (Algorithm 1, lines 12-15)
  const float lsum = sum_with_partner32(l);
  if (SPLIT) {  // partial result of this share of the keys, float32; no visible key: O = 0, L = -inf
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
    if (row_ok) {
      const long tok = si.tok0 + row;
      float* op = a.Opart + (((long)split * p.total_tokens + tok) * p.Hq + h) * D + 4 * hh;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 o;
#pragma unroll
          for (int u = 0; u < 4; ++u) o[u] = O[dt][4 * r4 + u] * inv;
          *(f32x4*)(op + 32 * dt + 8 * r4) = o;
        }
      if (hh == 0)
        a.Lpart[(long)split * p.total_tokens * p.Hq + s * p.lse_seq_stride + h * p.lse_head_stride + row] =
            lsum > 0.f ? m * p.scale + fast_log2(lsum) * kLn2 : -INFINITY;
    }
    return;
  }
  // (mask, window: a row without any key ends with l = 0: O = 0, L = -inf)
  const float inv = (MASK || LOCAL) && !(lsum > 0.f) ? 0.f : (DROPOUT ? p.drop_rp : 1.0f) / lsum;
  {
    // O through the ring slot that neither holds a block still in use nor receives one of the
    // copies issued past the last block (those fill the three slots after block ncol - 1)
    static_assert(RING == 4 && BUFB / 8 == 32 * D, "the staging area of a wavefront is an eighth of a ring slot");
    char* stg = smem + ((tend + 3) % RING) * BUFB + w * (BUFB / 8);
    __bf16* op = a.O + ((si.tok0 + prow0) * p.Hq + h) * dh;
    const long ostride = (long)p.Hq * dh;
    int ln = lane;  // recomputed here: nothing of the staging addresses is to live across the main loop
    asm volatile("" : "+v"(ln));
    if constexpr (DT % 2 == 0) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        store_rows_via_lds<DT / 2, F16>(stg, &O[half * (DT / 2)], inv, op + half * (DH / 2), ostride, n - prow0,
                                        dh - half * (DH / 2), ln);
      }
    } else {  // (an odd number of 32-column tiles: one at a time)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        store_rows_via_lds<1, F16>(stg, &O[dt], inv, op + 32 * dt, ostride, n - prow0, dh - 32 * dt, ln);
    }
    if (row < n && hh == 0)
      a.LSE[s * p.lse_seq_stride + h * p.lse_head_stride + (p.cu_seqlens ? si.tok0 : 0) + row] =
          MASK    ? (lsum > 0.f ? m + fast_log2(lsum) * kLn2 : -INFINITY)
          : LOCAL ? (lsum > 0.f ? m * p.scale + fast_log2(lsum) * kLn2 : -INFINITY)
                  : m * p.scale + fast_log2(lsum) * kLn2;
  }
}

// The same forward pass for a workgroup that takes `chain` items (row block, head, sequence)
// one after the other, d = 128, dense batches, no options. A workgroup's start-up (Q_i and the
// first two K/V tiles: a memory latency of several microseconds during which the matrix pipe
// idles) cannot be overlapped by a second resident workgroup here (128 KiB of LDS, 190
// registers), so the workgroup overlaps it with its own previous item: the three tile copies
// that every wavefront issues past an item's last block anyway fetch the NEXT item's first two
// tiles instead (the ring just keeps turning: an item's block j lives in slot (j + rb) % 4),
// and the next Q_i is requested into spare registers two blocks before the end. When the last
// barrier of an item falls, everything the next item's first phase reads is already in place.
//
// Items: an XCD's list is the one block_coord walks (under the mask heaviest row blocks
// first); workgroup k of the XCD's W takes positions k, 2W-1-k, 2W+k, 4W-1-k, ...: every
// workgroup gets the same amount of work whenever the chain length is even.
template <int D, bool CAUSAL, bool F16>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void fwd_chain_kernel(FwdArgs a, int chain) {
  constexpr int AHEAD_QK = kFwdAheadQK, AHEAD_PV = kFwdAheadPV;
  constexpr int BR = 256, BC = 64, RING = 4;
  constexpr int KS = D / 16, DT = D / 32, ROWB = 2 * D;
  constexpr int TILEB = BC * ROWB, BUFB = 2 * TILEB;  // one buffer = K_j | V_j

  __shared__ __attribute__((aligned(1024))) char smem[RING * BUFB];

  const Problem& p = a.p;
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = w >> 2;
  // Everything derived from the lane index is recomputed at the start of every item from a copy
  // the optimiser cannot see through: it would otherwise hoist the loop invariants of BOTH
  // groups' loops (LDS addresses by the dozen) out of the item loop, where they are all live at
  // once, and run out of registers.
  int lane = tid & 63, lq = lane & 31, hh = lane >> 5;
  // dense batch: every item has the same lengths
  const int n = p.N, nk = p.Nk, off = nk - n;
  const int nblk = (n + BR - 1) / BR;
  const int ncol_all = (nk + BC - 1) / BC;
  const long kstride = (long)p.Hkv * D, qstride = (long)p.Hq * D;

  // ---- items of this workgroup
  const int xcd = blockIdx.x % kXcds, kq = blockIdx.x / kXcds;
  const int wpx = gridDim.x / kXcds;            // workgroups per XCD
  const int ppx = p.Hq * p.nseq / kXcds;        // (head, sequence) pairs per XCD (the launch makes it exact)
  struct Item {
    const __bf16 *Kb, *Vb;
    int h, s, prow0, ncol;
  };
  auto locate = [&](int i) {
    const int pos = i * wpx + ((i & 1) ? wpx - 1 - kq : kq);
    int blk, pl;
    if (CAUSAL) {
      blk = pos / ppx;
      pl = pos % ppx;
    } else {
      blk = pos % nblk;
      pl = pos / nblk;
    }
    const int pr = pl * kXcds + xcd;
    Item it;
    const int hp = pr % p.Hq, nkv = p.Hq / p.G;  // heads of one group on one XCD (see block_coord)
    it.h = (hp % nkv) * p.G + hp / nkv;
    it.s = pr / p.Hq;
    const int i0 = (nblk - 1 - blk) * BR;
    it.prow0 = i0 + 32 * w;
    it.ncol = ncol_all;
    if (CAUSAL) {
      const int last_pos = (i0 + BR < n ? i0 + BR : n) - 1 + off;
      const int c = last_pos / BC + 1;
      it.ncol = c < ncol_all ? c : ncol_all;
    }
    const long kv = ((long)it.s * nk * p.Hkv + it.h / p.G) * D;
    it.Kb = a.K + kv;
    it.Vb = a.V + kv;
    return it;
  };
  auto q_address = [&](const Item& it) {
    const int row = it.prow0 + lq;
    const int rowc = row < n ? row : n - 1;  // rows past the end compute on a copy and are never stored
    return a.Q + (((long)it.s * n + rowc) * p.Hq + it.h) * D + 8 * hh;
  };

  Item cur = locate(0), nxt = cur;
  bool has_next = false;
  int rb = 0;       // ring slot of the current item's block 0
  int fwd_end = 0;  // blocks cur.ncol .. fwd_end - 1 of the current item are the next item's first blocks
  int jq = -8;      // the block after whose score product the next Q_i is requested: the item's last, if it has a successor

  u32x4 Qf[KS];
  {
    const __bf16* qp = q_address(cur);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Qf[ks] = *(const u32x4*)(qp + 16 * ks);
  }
  // The next item's Q_i goes straight into the registers of the current one, as soon as the
  // current item's last score product has been issued (its last matrix phase only updates O).
  auto request_next_q = [&]() {
    const __bf16* qp = q_address(nxt);
    load16_async<0>(Qf[0], qp);
    load16_async<32>(Qf[1], qp);
    load16_async<64>(Qf[2], qp);
    load16_async<96>(Qf[3], qp);
    if constexpr (KS == 8) {
      load16_async<128>(Qf[4], qp);
      load16_async<160>(Qf[5], qp);
      load16_async<192>(Qf[6], qp);
      load16_async<224>(Qf[7], qp);
    }
  };

  // Tile copies as in fwd_kernel (group 1 the K tiles, group 0 the V tiles, two blocks ahead,
  // exactly TPW copies per wavefront and vector phase). Blocks ncol and ncol + 1 of an item that
  // has a successor are the successor's blocks 0 and 1; block ncol + 2 (and every block past the
  // end of the last item) is a clamped copy that nobody reads.
  TileLoader<D, BC, 4, false> loader;
  loader.init(kstride, w & 3, lane, D / 8);
  int zrow, zcol[2];  // lane constants of the LDS addressing (see fa_lds.h)
  auto lane_constants = [&]() {
    lane = tid & 63;
    asm volatile("" : "+v"(lane));
    lq = lane & 31;
    hh = lane >> 5;
    loader.init(kstride, w & 3, lane, D / 8);
    zrow = lq * ROWB + 16 * (hh ^ swz<ROWB>(lq));
    const int p16 = lane & 15, g16 = (lane >> 4) & 1;
#pragma unroll
    for (int u = 0; u < 2; ++u)
      zcol[u] = swz_off<ROWB>(4 * hh + (p16 >> 2) + 8 * u, 2 * g16 + ((p16 & 3) >> 1)) + 8 * (p16 & 1);
  };
  constexpr int TPW = TileLoader<D, BC, 4, false>::PER;
  auto issue_tile = [&](int j) {
    char* dst = smem + ((j + rb) % RING) * BUFB + (grp == 0 ? TILEB : 0);
    const bool fwd_ = j >= cur.ncol && j < fwd_end;
    const __bf16* base = fwd_ ? (grp == 0 ? nxt.Vb : nxt.Kb) : (grp == 0 ? cur.Vb : cur.Kb);
    loader.load(dst, base, kstride, (fwd_ ? j - cur.ncol : j) * BC, nk - 1, w & 3, lane);
  };
  issue_tile(0);
  issue_tile(1);
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) touch(Qf[ks]);
  wait_vmem();
  lds_barrier();

  const float c2 = p.scale_log2e;

  // (one copy of the item loop per group, so that what the optimiser hoists out of one group's
  // loops is not live in the other's)
  auto run_items = [&](auto group) {
  constexpr int GRP = decltype(group)::value;
  for (int it = 0;; ++it) {
  f32x16 O[DT];
  float m, l;
  f32x16 S[2];
  bf16x8 Pf[2][2];
  int wrow_last, lim_row;  // position of the wavefront's last query among the keys; last visible column of this lane's row

  auto matrix_phase = [&](int j) {
    __builtin_amdgcn_s_setprio(FA_FWD_MATRIX_PRIO);
    if (j < cur.ncol && (!CAUSAL || j * BC <= wrow_last)) {  // S^T = K_j Q_i^T (Algorithm 1, line 8)
      const int zk = zrow + ((j + rb) % RING) * BUFB;
      S[0] = S[1] = (f32x16){0};
      mfma_stream<2 * KS, AHEAD_QK, 1>(
          [&](int i) { return lds_b128(smem, (zk ^ (32 * (i >> 1))) + (i & 1) * 32 * ROWB); },
          [&](int i, bf16x8 x) { S[i & 1] = mfma32<F16>(x, __builtin_bit_cast(bf16x8, Qf[i >> 1]), S[i & 1]); });
    }
    if (j > 0 && (!CAUSAL || (j - 1) * BC <= wrow_last)) {  // O^T += V_{j-1}^T P^T (line 10)
      const int vb = ((j - 1 + rb) % RING) * BUFB + TILEB;
      const int zv0 = zcol[0] + vb, zv1 = zcol[1] + vb;
      mfma_stream<4 * DT, AHEAD_PV, 2>(
          [&](int i) {
            const int dt = i >> 2, ro = (16 * (i & 3)) * ROWB;
            return lds_tr_pair(smem, (zv0 ^ (64 * dt)) + ro, (zv1 ^ (64 * dt)) + ro);
          },
          [&](int i, bf16x8 x) { O[i >> 2] = mfma32<F16>(x, Pf[(i >> 1) & 1][i & 1], O[i >> 2]); });
    }
    __builtin_amdgcn_s_setprio(0);
  };

  auto vector_phase = [&](int j) {  // online softmax of block j (line 9), as in fwd_kernel
    if (j >= cur.ncol || (CAUSAL && j * BC > wrow_last)) return;
    const int col0 = j * BC;
    const bool need_mask = (CAUSAL && col0 + BC - 1 > cur.prow0 + off) || (col0 + BC > nk);
    if (need_mask) {
      asm volatile("; keep this a branch: the mask costs two instructions per element" ::);
      const int lim = lim_row - col0 - 4 * hh;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) S[kt][r] = 32 * kt + acc_row(r, 0) > lim ? -INFINITY : S[kt][r];
    }
    // (fast path without the row maximum, see fwd_kernel)
    float rs0, rs1;
    auto exponentials = [&](float ref) {
      rs0 = rs1 = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        f32x16 E;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          E[r] = fast_exp2(__builtin_fmaf(S[kt][r], c2, -ref));
          E[r + 1] = fast_exp2(__builtin_fmaf(S[kt][r + 1], c2, -ref));
          rs0 += E[r];
          rs1 += E[r + 1];
        }
        Pf[kt][0] = pack8<F16>(E, 0);
        Pf[kt][1] = pack8<F16>(E, 1);
      }
    };
    bool advance = j == 0;
    if (!advance) {
      exponentials(m * c2);
      advance = __builtin_amdgcn_ballot_w64(rs0 + rs1 > (float)(1 << (F16 ? kFwdLazyLog2Half : kFwdLazyLog2Bf16))) != 0;
    }
    if (advance) {
      float mx = max3(S[0][0], S[0][1], S[1][0]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = max3(mx, S[0][r], S[0][r + 1]);
      mx = max3(mx, S[1][1], S[1][2]);
      mx = fmaxf(mx, S[1][3]);
#pragma unroll
      for (int r = 4; r < 16; r += 2) mx = max3(mx, S[1][r], S[1][r + 1]);
      mx = max_with_partner32(mx);
      const float m_new = fmaxf(m, mx);
      const float alpha = fast_exp2((m - m_new) * c2);
      l *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
      m = m_new;
      exponentials(m * c2);
    }
    l += rs0 + rs1;
  };

    lane_constants();
    has_next = it + 1 < chain;
    if (has_next) nxt = locate(it + 1);
    const int ncol = cur.ncol;
    // (kept as numbers compared with j rather than as flags, and opaque to the optimiser: it would
    // otherwise build every loop twice, with and without a successor, and run out of registers)
    fwd_end = has_next ? ncol + 2 : ncol;
    jq = has_next ? ncol - 1 : -8;
    asm volatile("" : "+s"(fwd_end), "+s"(jq));
    {
      const int row = cur.prow0 + lq;
      wrow_last = cur.prow0 + 31 + off;
      lim_row = CAUSAL ? (row + off < nk - 1 ? row + off : nk - 1) : nk - 1;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x16){0};
    m = -INFINITY;
    l = 0.f;

    // Phases as in fwd_kernel. Per wavefront the copies end in the order: block ncol + 1 (the
    // next item's block 1), the KS loads of the next Q_i, block ncol + 2 (read by nobody). The
    // waits of the last two blocks let the newer of these stay in flight; the wait after the last
    // barrier completes all but the newest TPW, i.e. everything the next item reads.
    constexpr int LATE = 2 * TPW + KS;
    // (one barrier per block, as in fwd_kernel's one-workgroup form: the barriers that followed no
    // wait are left out)
    if constexpr (GRP == 0) {
      for (int j = 0; j <= ncol; ++j) {
        matrix_phase(j);
        issue_tile(j + 2);
        if (j == jq) request_next_q();
        vector_phase(j);
        if (j == jq) wait_vmem_upto<TPW + KS>();
        else if (j == jq + 1) wait_vmem_upto<LATE>();
        else wait_vmem_upto<TPW>();
        lds_barrier();
      }
    } else {
      issue_tile(2);
      for (int j = 0; j <= ncol; ++j) {
        matrix_phase(j);
        if (j == jq + 1) wait_vmem_upto<LATE>();
        else wait_vmem_upto<TPW>();
        lds_barrier();
        if (j < ncol) {
          if (j == jq) request_next_q();
          issue_tile(j + 3);
          vector_phase(j);
        }
      }
    }
    wait_vmem_upto<TPW>();

    // ---- epilogue of this item (lines 12-15); the next item's first tiles and Q_i are in place
    {
      const float lsum = sum_with_partner32(l);
      const float inv = 1.0f / lsum;
      char* stg = smem + ((ncol + 3 + rb) % RING) * BUFB + w * (BUFB / 8);
      __bf16* op = a.O + (((long)cur.s * n + cur.prow0) * p.Hq + cur.h) * D;
#pragma unroll
      for (int half = 0; half < 2; ++half)
        store_rows_via_lds<DT / 2, F16>(stg, &O[half * (DT / 2)], inv, op + half * (D / 2), qstride, n - cur.prow0, D / 2, lane);
      const int row = cur.prow0 + lq;
      if (row < n && hh == 0)
        a.LSE[cur.s * p.lse_seq_stride + cur.h * p.lse_head_stride + row] = m * p.scale + fast_log2(lsum) * kLn2;
    }
    // (before the exit test, so that in the compiler's output every path from the loads of the
    // next Q_i passes this point: that is what the host-side check of the assembly relies on)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) landed(Qf[ks]);
    if (!has_next) break;
    rb = (rb + ncol) % RING;
    cur = nxt;
  }
  };
  if (grp == 0) run_items(std::integral_constant<int, 0>{});
  else run_items(std::integral_constant<int, 1>{});
}

// Combine the partial results of the key shares: one thread per 4 output elements.
template <int D, bool F16>
__global__ __launch_bounds__(256) void fwd_merge_kernel(FwdArgs a) {
  constexpr int TPR = D / 4;  // threads per (token, head) row
  const Problem& p = a.p;
  const long nrows = (long)p.total_tokens * p.Hq;
  const long r = (long)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
  if (r >= nrows) return;
  const int c = threadIdx.x % TPR;
  const long tok = r / p.Hq;
  const int h = (int)(r - tok * p.Hq);
  const long b = tok / p.N, q = tok - b * p.N;
  const long li = b * p.lse_seq_stride + (long)h * p.lse_head_stride + q;
  // (a cache without keys: the split kernel wrote nothing for this sequence)
  const bool keyless = a.seqlens_k && a.seqlens_k[b] <= 0;
  float mx = -INFINITY;
  if (!keyless)
    for (int k = 0; k < a.nsplit; ++k) mx = fmaxf(mx, a.Lpart[(long)k * nrows + li]);
  if (mx == -INFINITY) {  // no share holds a key that this row sees: P = 0, so O = 0 and L = -inf
    *(u32x2*)(a.O + r * D + 4 * c) = (u32x2){0u, 0u};
    if (c == 0) a.LSE[li] = -INFINITY;
    return;
  }
  float z = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < a.nsplit; ++k) {
    const float lp = a.Lpart[(long)k * nrows + li];
    if (lp == -INFINITY) continue;  // a share without keys for this row (it may have written no partial O at all)
    const float wgt = __expf(lp - mx);
    const f32x4 o = *(const f32x4*)(a.Opart + ((long)k * nrows + r) * D + 4 * c);
    z += wgt;
    acc += o * wgt;
  }
  const float inv = 1.f / z;  // some share holds a visible key
  u32x2 o;
  o[0] = pack2<F16>(acc[0] * inv, acc[1] * inv);
  o[1] = pack2<F16>(acc[2] * inv, acc[3] * inv);
  *(u32x2*)(a.O + r * D + 4 * c) = o;
  if (c == 0) a.LSE[li] = mx + __logf(z);
}

// A sequence without any key (possible in ragged batches with two lengths) has no softmax. Its
// query rows get what rows emptied by an elementwise mask get: P = 0, hence O = 0 (and dQ = 0)
// and L = -inf. The attention kernels skip such sequences; this one, launched beside them for
// ragged batches with two lengths, fills their rows: one workgroup per sequence, the rows of a
// sequence being one contiguous piece of the token-major tensor. `lse` may be nullptr (dQ).
__global__ __launch_bounds__(256) void keyless_rows_kernel(Problem p, __bf16* out, float* lse) {
  const SeqInfo si = seq_info(p, blockIdx.x);
  if (si.nk != 0 || si.n == 0) return;
  u32x4* o = (u32x4*)(out + si.tok0 * p.Hq * p.d);
  const long chunks = (long)si.n * p.Hq * p.d / 8;
  for (long i = threadIdx.x; i < chunks; i += 256) o[i] = (u32x4){0, 0, 0, 0};
  if (lse)
    for (long i = threadIdx.x; i < (long)si.n * p.Hq; i += 256)
      lse[(i / si.n) * p.lse_head_stride + si.tok0 + i % si.n] = -INFINITY;
}
hipError_t launch_keyless_rows(const Problem& p, __bf16* out, float* lse, hipStream_t st) {
  if (!p.cu_seqlens_k) return hipSuccess;  // one length per sequence: a sequence with queries has keys
  hipLaunchKernelGGL(keyless_rows_kernel, dim3(p.nseq), dim3(256), 0, st, p, out, lse);
  return hipGetLastError();
}

template <int D, bool F16>
static hipError_t launch_fwd_d(const FwdArgs& a, int causal, hipStream_t st) {
  dim3 block(512);
  if (a.nsplit > 0) {
    if (a.p.N * a.p.G <= 32) {  // one row tile per key/value head: the wavefronts divide the keys (fa_decode.hip)
      if (hipError_t e = launch_fwd_decode(a, D, causal, st)) return e;
      if (a.nsplit == 1) return hipSuccess;  // (a single share: that kernel has written O and LSE itself)
    } else {
      const int nblk = (a.p.N * a.p.G + 255) / 256;
      dim3 grid(grid_size(nblk * a.nsplit, a.p.Hkv * a.p.nseq));
      if (causal) hipLaunchKernelGGL((fwd_kernel<D, true, true, F16>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((fwd_kernel<D, false, true, F16>), grid, block, 0, st, a);
      if (hipError_t e = hipGetLastError()) return e;
    }
    constexpr int RPB = 256 / (D / 4);
    const long nrows = (long)a.p.total_tokens * a.p.Hq;
    hipLaunchKernelGGL((fwd_merge_kernel<D, F16>), dim3((unsigned)((nrows + RPB - 1) / RPB)), dim3(256), 0, st, a);
    return hipGetLastError();
  }
  dim3 grid(grid_size((a.p.N + 255) / 256, a.p.Hq * a.p.nseq));
  if (a.p.mask) {  // the entry points keep everything else away from it
    if (causal) hipLaunchKernelGGL((fwd_kernel<D, true, false, F16, false, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((fwd_kernel<D, false, false, F16, false, false, true>), grid, block, 0, st, a);
    return hipGetLastError();
  }
  if (a.p.win_left >= 0 || a.p.win_right >= 0 || a.p.bmask) {  // sliding window, block-sparse pattern (the entry points keep everything else away from them)
    hipLaunchKernelGGL((fwd_kernel<D, false, false, F16, false, false, false, true>), grid, block, 0, st, a);
    return hipGetLastError();
  }
  if (a.p.d != D) {  // padded head dimension (the entry points keep dropout away from it)
    constexpr int DN = D == 128 ? 96 : 32;  // the narrower product width of this tile width
    if (a.p.d <= DN) {
      if (causal) hipLaunchKernelGGL((fwd_kernel<D, true, false, F16, false, true, false, false, DN>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((fwd_kernel<D, false, false, F16, false, true, false, false, DN>), grid, block, 0, st, a);
    } else {
      if (causal) hipLaunchKernelGGL((fwd_kernel<D, true, false, F16, false, true>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((fwd_kernel<D, false, false, F16, false, true>), grid, block, 0, st, a);
    }
    return hipGetLastError();
  }
  if (a.p.drop_thr) {
    if (causal) hipLaunchKernelGGL((fwd_kernel<D, true, false, F16, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((fwd_kernel<D, false, false, F16, true>), grid, block, 0, st, a);
    return hipGetLastError();
  }
  if constexpr (D == 128) {
    // chained items (fwd_chain_kernel): dense batches of short sequences (at most 16 key blocks:
    // +15% at N = 512; from N = 2048 on the start-up no longer matters and the fixed assignment
    // of items loses against the hardware's dynamic one, -5% at N = 8192 under the mask) whose
    // items split evenly over the XCDs and into chains of even length, with at least one
    // workgroup left per compute unit
    const int pairs = a.p.Hq * a.p.nseq, nblk = (a.p.N + 255) / 256;
    if (!a.p.cu_seqlens && pairs % kXcds == 0 && a.p.N >= 256 && a.p.Nk >= a.p.N && a.p.Nk <= kFwdChainMaxN) {
      const int items = pairs / kXcds * nblk;  // per XCD
      int chain = items % 8 == 0 ? 8 : items % 4 == 0 ? 4 : items % 2 == 0 ? 2 : 1;
      while (chain > 1 && items / chain < 32) chain /= 2;
      if (chain > 1) {
        dim3 cgrid((unsigned)(kXcds * (items / chain)));
        if (causal) hipLaunchKernelGGL((fwd_chain_kernel<D, true, F16>), cgrid, block, 0, st, a, chain);
        else hipLaunchKernelGGL((fwd_chain_kernel<D, false, F16>), cgrid, block, 0, st, a, chain);
        return hipGetLastError();
      }
    }
  }
  if (causal) hipLaunchKernelGGL((fwd_kernel<D, true, false, F16>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((fwd_kernel<D, false, false, F16>), grid, block, 0, st, a);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdArgs& a, int d, int causal, hipStream_t st) {
  if (hipError_t e = launch_keyless_rows(a.p, a.O, a.LSE, st)) return e;
  if (d == 256) return launch_fwd256(a, causal, st);
  // tile width: the head dimension padded up to 64 or 128
  if (a.p.f16) return d <= 64 ? launch_fwd_d<64, true>(a, causal, st) : launch_fwd_d<128, true>(a, causal, st);
  return d <= 64 ? launch_fwd_d<64, false>(a, causal, st) : launch_fwd_d<128, false>(a, causal, st);
}

}  // namespace fa
