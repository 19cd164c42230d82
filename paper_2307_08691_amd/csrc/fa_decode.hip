// Forward for very few query rows against many keys (decoding: one or a few new tokens per
// sequence against a key/value cache; the inference setting of the multi-query / grouped-query
// paragraph of section 3.1). Algorithm 1 with the parallelism turned round: the rows of one
// (sequence, key/value head) — query row x query head of the group, at most 32 — fit ONE 32-row
// MFMA tile, so there is nothing to split over wavefronts along the rows. Instead the eight
// wavefronts of a workgroup take the KEY tiles (32 keys each) of the workgroup's share of the keys
// in turn, every wavefront with a running softmax of its own (m, l, O), without a barrier inside
// the loop; at the end the eight partial results are combined through LDS with the identity the
// paper uses between blocks (section 3.1.1) and the workgroup writes its share's normalised
// partial O and logsumexp, which fwd_merge_kernel combines over the shares as for the split kernel.
// The pass is bound by HBM: K and V are read once, and the point of the layout is to keep eight
// independent streams of loads in flight per compute unit.
//
// Per 32-key tile and wavefront: K_j goes straight from memory into the A-operand registers of
// S^T = K_j Q^T (lane (key, half) fetches 16 bytes of its key's row per contraction step), V_j goes
// memory -> LDS by direct copies into a tile private to the wavefront and is read back transposed
// as the A operand of O^T += V_j^T P^T. Both are requested one tile ahead (two register sets,
// two LDS tiles per wavefront). The K loads are ordinary loads (the compiler waits for them where
// they are used); the V copies are the hand-issued direct-to-LDS copies of fa_lds.h, which the
// compiler does not see: one s_waitcnt vmcnt(0) per tile, after the tile's work, covers them.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "fa_kernels.h"
#include "fa_lds.h"

namespace fa {

template <int D, bool CAUSAL, bool F16>
__global__ __launch_bounds__(512) void fwd_decode_kernel(FwdArgs a) {
  constexpr int KT = 32;             // keys per tile
  constexpr int KS = D / 16;         // contraction steps of the first product
  constexpr int DT = D / 32;         // 32-row tiles of O^T
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = KT * ROWB;   // one V tile
  constexpr int WAVEB = 2 * TILEB;   // a wavefront's two V tiles; later its partial O^T (D x 32 floats)
  static_assert(WAVEB == D * 32 * 4, "the partial O^T of a wavefront takes the place of its two V tiles");
  constexpr int STAT_OFF = 8 * WAVEB;  // m and l of the eight wavefronts: [2][8][32] floats
  __shared__ __attribute__((aligned(1024))) char smem[STAT_OFF + 2 * 8 * 32 * 4];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, hh = lane >> 5;
  const int nsplit = a.nsplit;
  const BlockCoord bc = block_coord<false>(nsplit, p.Hkv, p.nseq);
  if (!bc.valid) return;
  const int split = bc.blk, g = bc.head;
  // Sequences of uneven cache lengths are handed out longest first: the workgroups of an XCD take
  // their (sequence, head) pairs in launch order, and a long sequence that starts last leaves the
  // other compute units idle at the end. bc.seq is therefore read as a RANK, and the sequence of that
  // rank (by length, ties by index) is found here: lane c counts the sequences that come before
  // candidate c. Done by every wavefront for itself (a few hundred scalar loads that hit L2); batches
  // of more than kRankMax sequences keep the launch order.
  constexpr int kRankMax = 128;
  int s_ = bc.seq;
  if (a.seqlens_k && p.nseq > 1 && p.nseq <= kRankMax) {
    auto len_of = [&](int i) {
      const int len = a.seqlens_k[i];
      return len < 0 ? 0 : (len < p.Nk ? len : p.Nk);
    };
    int found = 0;
    for (int c0 = 0; c0 < p.nseq; c0 += 64) {
      const int c = c0 + lane;
      const int lc = c < p.nseq ? len_of(c) : -1;
      int before = 0;
      for (int j = 0; j < p.nseq; ++j) {
        const int lj = __builtin_amdgcn_readfirstlane(len_of(j));
        before += (lj > lc || (lj == lc && j < c)) ? 1 : 0;
      }
      const unsigned long long hit = __builtin_amdgcn_ballot_w64(c < p.nseq && before == bc.seq);
      if (hit) found = c0 + __builtin_ctzll(hit);
    }
    s_ = found;
  }
  const int s = __builtin_amdgcn_readfirstlane(s_);
  const SeqInfo si = seq_info(p, s);
  int nk_ = si.nk;
  if (a.seqlens_k) {  // a key/value cache filled up to a length of its own per sequence
    const int len = a.seqlens_k[s];
    nk_ = len < 0 ? 0 : (len < p.Nk ? len : p.Nk);
  }
  const int n = si.n, nk = nk_;
  // With a single share there is nothing to merge: the workgroup writes O and LSE themselves (and
  // the launch leaves fwd_merge_kernel out), also for a sequence without keys.
  const bool direct = nsplit == 1;
  if (n == 0) return;
  if (nk == 0) {  // (several shares: fwd_merge_kernel fills the rows)
    if (direct) {
      for (int i = tid; i < n * p.G * (D / 8); i += 512) {  // 16-byte pieces of the rows of this key/value head
        const int prow_ = i / (D / 8), q_ = prow_ / p.G, h_ = g * p.G + prow_ % p.G;
        *(u32x4*)(a.O + ((si.tok0 + q_) * p.Hq + h_) * D + 8 * (i % (D / 8))) = (u32x4){0, 0, 0, 0};
        if (i % (D / 8) == 0) a.LSE[s * p.lse_seq_stride + (long)h_ * p.lse_head_stride + q_] = -INFINITY;
      }
    }
    return;
  }
  const int off = nk - n;
  const int nrows = n * p.G;  // packed rows: query * G + head of the group; at most 32 (the launch checks)

  // this lane's packed row, its query and its head
  const bool row_ok = lq < nrows;
  const int prow = row_ok ? lq : nrows - 1;  // lanes past the end compute on a copy and store nothing
  const int row = prow / p.G, h = g * p.G + prow % p.G;
  bf16x8 Qf[KS];
  {
    const __bf16* qp = a.Q + ((si.tok0 + row) * p.Hq + h) * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Qf[ks] = *(const bf16x8*)(qp + 16 * ks);
  }

  // the share's keys, in blocks of 64 as in the split kernel (the two kernels split alike), then in tiles of 32
  const int ncol_all = (nk + 63) / 64;
  const int per_split = (ncol_all + nsplit - 1) / nsplit;
  const int jb = split * per_split;
  const int ncol = jb + per_split < ncol_all ? jb + per_split : ncol_all;  // (the last query stands at the last key: no causal bound)
  const long lpart = (long)split * p.total_tokens * p.Hq + s * p.lse_seq_stride + (long)h * p.lse_head_stride + row;
  if (jb >= ncol) {  // no key of this share is visible: L = -inf says so to the merge
    if (w == 0 && row_ok && hh == 0) a.Lpart[lpart] = -INFINITY;
    return;
  }
  const int t_begin = 2 * jb, t_end = (nk + KT - 1) / KT < 2 * ncol ? (nk + KT - 1) / KT : 2 * ncol;  // tiles of 32 keys

  // ---- loads of one tile: K rows into registers, V rows into the wavefront's LDS tile `buf`
  const long kstride = (long)p.Hkv * D;
  char* vbuf = smem + w * WAVEB;
  u32x4 Kr[2][KS];
  const int pmask = a.block_table ? (1 << a.page_log2) - 1 : 0;
  auto tile_base = [&](int t, const __bf16* pool, int& first, int& last) {  // rows of tile t: base pointer, first row, last valid row
    const int key0 = t * KT;
    if (a.block_table) {
      const int in_page = key0 & pmask;
      const int pg = __builtin_amdgcn_readfirstlane(a.block_table[(long)s * a.table_stride + (key0 >> a.page_log2)]);
      first = in_page;
      last = nk - 1 - (key0 - in_page);
      last = last < pmask ? last : pmask;
      return pool + (((long)pg << a.page_log2) * p.Hkv + g) * D;
    }
    first = key0;
    last = nk - 1;
    return pool + (si.tok0k * p.Hkv + g) * D;
  };
  auto issue = [&](int t, auto BUF) {
    constexpr int buf = decltype(BUF)::value;
    int first, last;
    const __bf16* kb = tile_base(t, a.K, first, last);
    const int kr = first + lq < last ? first + lq : last;  // keys past the end repeat the last one (masked below)
    const __bf16* kp = kb + (long)kr * kstride + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Kr[buf][ks] = *(const u32x4*)(kp + 16 * ks);
    const __bf16* vb = tile_base(t, a.V, first, last);
    tile_load_async<D, KT, 1>(vbuf + buf * TILEB, vb, kstride, first, last, 0, lane);
  };

  // ---- on-chip state of this wavefront (Algorithm 1, line 5)
  f32x16 O[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) O[dt] = (f32x16){0};
  float m = -INFINITY, l = 0.f;
  const float c2 = p.scale_log2e;
  const int pos = row + off;  // this lane's query among the keys

  // lane constants of the transposing V reads (see fa_lds.h)
  const int p16 = lane & 15, g16 = (lane >> 4) & 1;
  int zcol[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
    zcol[u] = swz_off<ROWB>(4 * hh + (p16 >> 2) + 8 * u, 2 * g16 + ((p16 & 3) >> 1)) + 8 * (p16 & 1);

  auto compute = [&](int t, auto BUF) {
    constexpr int buf = decltype(BUF)::value;
    // ---- S^T = K_j Q^T (Algorithm 1, line 8)
    f32x16 S = (f32x16){0};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) S = mfma32<F16>(__builtin_bit_cast(bf16x8, Kr[buf][ks]), Qf[ks], S);
    // ---- keys past the end and (causal) above the query's position
    const int key0 = t * KT;
    const int lim = (CAUSAL && pos < nk - 1 ? pos : nk - 1) - key0 - 4 * hh;  // last visible key, relative to this lane's first
    if (key0 + KT - 1 > (CAUSAL ? off : nk - 1) || key0 + KT > nk) {
#pragma unroll
      for (int r = 0; r < 16; ++r) S[r] = acc_row(r, 0) > lim ? -INFINITY : S[r];
    }
    // ---- online softmax (Algorithm 1, line 9); a row may have seen no key yet
    float mx = S[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S[r]);
    mx = max_with_partner32(mx);
    const float m_new = fmaxf(m, mx);
    const float alpha = m_new == -INFINITY ? 1.f : fast_exp2((m - m_new) * c2);
    const float ref = m_new == -INFINITY ? 0.f : m_new * c2;
    float rs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      S[r] = fast_exp2(__builtin_fmaf(S[r], c2, -ref));
      rs += S[r];
    }
    l = l * alpha + rs;
    m = m_new;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
    bf16x8 Pf[2];
    Pf[0] = pack8<F16>(S, 0);
    Pf[1] = pack8<F16>(S, 1);
    // ---- O^T += V_j^T P^T (Algorithm 1, line 10)
    const int vb = w * WAVEB + buf * TILEB;
#pragma unroll
    for (int i = 0; i < 2 * DT; ++i) {
      const int dt = i >> 1, ro = (16 * (i & 1)) * ROWB;
      const bf16x8 x = lds_tr_pair(smem, ((zcol[0] + vb) ^ (64 * dt)) + ro, ((zcol[1] + vb) ^ (64 * dt)) + ro);
      O[dt] = mfma32<F16>(x, Pf[i & 1], O[dt]);
    }
  };

  // ---- this wavefront's tiles: t_begin + w, + 8, ...; the next one is requested before the current one is used
  using B0 = std::integral_constant<int, 0>;
  using B1 = std::integral_constant<int, 1>;
  int t = t_begin + w;
  if (t < t_end) {
    issue(t, B0{});
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) touch(Qf[ks]);
    wait_vmem();
    while (true) {
      if (t + 8 < t_end) issue(t + 8, B1{});
      compute(t, B0{});
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the reads of this tile are done before its buffer is requested again
      wait_vmem();
      t += 8;
      if (t >= t_end) break;
      if (t + 8 < t_end) issue(t + 8, B0{});
      compute(t, B1{});
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      wait_vmem();
      t += 8;
      if (t >= t_end) break;
    }
  }

  // ---- combine the eight wavefronts (section 3.1.1's rescaling, once more) and write the share's partial result
  const float lsum = sum_with_partner32(l);
  __syncthreads();  // every wavefront is done with its V tiles
  float* part = (float*)(smem + w * WAVEB);  // [d][row]
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) part[(32 * dt + acc_row(r, hh)) * 32 + lq] = O[dt][r];
  float* stat = (float*)(smem + STAT_OFF);
  if (hh == 0) {
    stat[w * 32 + lq] = m;
    stat[256 + w * 32 + lq] = lsum;
  }
  __syncthreads();
  {
    const int r = tid & 31, dg = tid >> 5;  // this thread: row r, columns dg * (D / 16) ..
    float mm = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < 8; ++ww) mm = fmaxf(mm, stat[ww * 32 + r]);
    float wgt[8], den = 0.f;
#pragma unroll
    for (int ww = 0; ww < 8; ++ww) {
      const float mw = stat[ww * 32 + r];
      wgt[ww] = mw == -INFINITY ? 0.f : fast_exp2((mw - mm) * c2);
      den += wgt[ww] * stat[256 + ww * 32 + r];
    }
    const bool ok = r < nrows;
    const int prow2 = ok ? r : nrows - 1;
    const int row2 = prow2 / p.G, h2 = g * p.G + prow2 % p.G;
    const float inv = den > 0.f ? 1.f / den : 0.f;  // no visible key in this share: O = 0, L = -inf
    float out[D / 16];
#pragma unroll
    for (int i = 0; i < D / 16; ++i) {
      const int dcol = dg * (D / 16) + i;
      float acc = 0.f;
#pragma unroll
      for (int ww = 0; ww < 8; ++ww) acc += wgt[ww] * ((const float*)(smem + ww * WAVEB))[dcol * 32 + r];
      out[i] = acc * inv;
    }
    const float lse = den > 0.f ? mm * p.scale + fast_log2(den) * kLn2 : -INFINITY;
    const long lidx = s * p.lse_seq_stride + (long)h2 * p.lse_head_stride + row2;
    if (direct) {  // the final result, rounded to the element type
      if (ok) {
        __bf16* op = a.O + ((si.tok0 + row2) * p.Hq + h2) * D + dg * (D / 16);
        if constexpr (D == 128) {  // eight columns: 16 bytes
          u32x4 v;
#pragma unroll
          for (int u = 0; u < 4; ++u) v[u] = pack2<F16>(out[2 * u], out[2 * u + 1]);
          *(u32x4*)op = v;
        } else {  // four columns: 8 bytes
          u32x2 v;
          v[0] = pack2<F16>(out[0], out[1]);
          v[1] = pack2<F16>(out[2], out[3]);
          *(u32x2*)op = v;
        }
        if (dg == 0) a.LSE[lidx] = lse;
      }
    } else if (ok) {
      float* op = a.Opart + (((long)split * p.total_tokens + si.tok0 + row2) * p.Hq + h2) * D + dg * (D / 16);
#pragma unroll
      for (int i = 0; i < D / 16; ++i) op[i] = out[i];
      if (dg == 0) a.Lpart[(long)split * p.total_tokens * p.Hq + lidx] = lse;
    }
  }
}

// `a.nsplit` shares per (sequence, key/value head); N * G <= 32 rows. The caller runs fwd_merge_kernel afterwards.
template <int D>
static hipError_t launch_decode_d(const FwdArgs& a, int causal, hipStream_t st) {
  dim3 grid(grid_size(a.nsplit, a.p.Hkv * a.p.nseq)), block(512);
  if (a.p.f16) {
    if (causal) hipLaunchKernelGGL((fwd_decode_kernel<D, true, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((fwd_decode_kernel<D, false, true>), grid, block, 0, st, a);
  } else {
    if (causal) hipLaunchKernelGGL((fwd_decode_kernel<D, true, false>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((fwd_decode_kernel<D, false, false>), grid, block, 0, st, a);
  }
  return hipGetLastError();
}

hipError_t launch_fwd_decode(const FwdArgs& a, int d, int causal, hipStream_t st) {
  if (d == 64) return launch_decode_d<64>(a, causal, st);
  if (d == 128) return launch_decode_d<128>(a, causal, st);
  return hipErrorInvalidValue;
}

}  // namespace fa
