// Forward pass of exact attention on FP8 (OCP E4M3) operands for gfx950 (Algorithm 1 of the
// paper; section 5 names FP8 as a direction, the convention is this library's: see fa.h).
//
// Same skeleton as fwd_kernel: one workgroup (8 wavefronts) owns 256 query rows, each wavefront 32
// whole rows; scores are computed transposed, S^T = K_j Q_i^T, so the softmax reductions stay
// inside a lane; matrix and vector phases separated by barriers, the two wave groups one phase
// apart; K_j and V_j^T stream HBM -> LDS two blocks ahead into a ring of four buffers.
//
// What differs is the matrix instruction, v_mfma_f32_32x32x64_f8f6f4: 64 contraction elements per
// instruction, a lane supplying 32 consecutive bytes of its row (A) or column (B). Both operands
// of a product are filled by the same rule (lane half hh, register j, byte b <-> one contraction
// index), so the sums are right whatever order the hardware takes the indices in.
//  * S^T = K_j Q_i^T contracts over the head dimension: A = 32 bytes of a K row from LDS, B = 32
//    bytes of the lane's Q row from registers.
//  * O^T += V_j^T P^T contracts over the 64 keys of the block in ONE instruction per 32 rows of
//    O^T. B must hold a lane's 32 exponentials as bytes in the order of its accumulator registers;
//    A must hold V^T[d][key] for the same keys in the same order. The rows of the K tile are
//    therefore assigned to accumulator rows by a permutation under which a lane half holds two
//    runs of 16 CONSECUTIVE keys: accumulator row 8q + 4h + u of tile kt stands for key
//    32 kt + 16 h + 4 q + u. V arrives key-major (V^T[d][key], rows padded to 64 keys), so A is
//    two plain 16-byte reads per tile; nothing is transposed on chip.
//  * P = exp(S - m) * 2^8 is rounded to E4M3 (v_cvt_pk_fp8_f32), m the true running maximum, so
//    the operand stays below 448 and resolves P down to 2^-17 of the row's maximum; the row sum
//    is taken from the float32 exponentials.
#include "fa_common.h"
#include "fa_kernels.h"
#include "fa_lds.h"

namespace fa {

typedef __attribute__((ext_vector_type(8))) int i32x8;

// 16-byte chunk swizzles (XOR on the chunk index inside a row) under which the operand reads below
// are conflict free. K tile, rows of ROWB bytes: the 16 lanes of a read group fetch the same chunk
// of rows {a .. a+3, a+16 .. a+19, a+4 .. a+7, a+20 .. a+23} (the permutation above).
template <int ROWB>
__device__ __forceinline__ int swz_k8(int row) {
  if (ROWB == 128) return ((row >> 1) & 1) | (((row >> 2) & 1) << 1) | (((row >> 4) & 1) << 2);  // 2 rows per 256 bytes
  return ((row >> 2) & 1) | (((row >> 4) & 1) << 1);                                              // 64-byte rows: 4 per 256
}
// V^T tile, rows of 64 bytes (64 keys), one row per head-dimension index: 16 consecutive rows per read group
__device__ __forceinline__ int swz_v8(int row) { return (row >> 2) & 3; }

__device__ __forceinline__ i32x8 join(u32x4 lo, u32x4 hi) {
  return (i32x8){(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
}

__device__ __forceinline__ f32x16 mfma_fp8(i32x8 a, i32x8 b, f32x16 c) {
  // (format selectors 0, 0: both operands E4M3; scales 0: the unscaled instruction)
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
}

// (d = 64: 32 KiB of LDS and fewer than 128 registers, so two workgroups share a compute unit and one's
// start-up and epilogue overlap the other's loop, as in the bf16 kernel)
template <int D, bool CAUSAL>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(D == 64 ? 4 : 2, D == 64 ? 4 : 2))) void fwd_fp8_kernel(Fp8Args a) {
  constexpr int BR = 256, BC = 64, RING = 4;
  constexpr int KS = D / 64;   // contraction steps of the first product
  constexpr int DT = D / 32;   // 32-row tiles of O^T
  constexpr int KROWB = D;     // bytes of a K row
  constexpr int KTILE = BC * KROWB, VTILE = D * BC, BUFB = KTILE + VTILE;  // one buffer = K_j | V_j^T
  constexpr int KCPR = KROWB / 16, KRPI = 64 / KCPR;  // chunks per K row, K rows per copy instruction
  constexpr int TPW = KTILE / 1024 / 4;               // copies per wavefront per tile (K and V^T tiles are the same size)
  static_assert(KTILE == VTILE && TPW >= 1, "both tiles take the same number of copies");

  __shared__ __attribute__((aligned(1024))) char smem[RING * BUFB];

  const Problem& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = w >> 2;
  const int lq = lane & 31, hh = lane >> 5;
  const int nblk = (p.N + BR - 1) / BR;
  const BlockCoord bc = block_coord<CAUSAL>(nblk, p.Hq, p.nseq, p.G);
  if (!bc.valid) return;
  const int rowblk = nblk - 1 - bc.blk;  // longest causal rows first
  const int s = bc.seq, h = bc.head, g = h / p.G;
  const int n = p.N, nk = p.Nk, off = nk - n;
  const int i0 = rowblk * BR;
  if (i0 >= n) return;
  const long kstride = (long)p.Hkv * D;                                  // bytes between K rows
  const char* Kb = (const char*)a.K + ((long)s * nk * p.Hkv + g) * D;
  const char* Vb = (const char*)a.Vt + ((long)s * p.Hkv + g) * D * a.vt_stride;  // row = head-dimension index

  // ---- Q_i operands: 32 bytes per contraction step (Algorithm 1, line 4)
  const int prow0 = i0 + 32 * w, row = prow0 + lq;
  const int rowc = row < n ? row : n - 1;  // rows past the end compute on a copy and are never stored
  i32x8 Qf[KS];
  {
    const char* qp = (const char*)a.Q + (((long)s * n + rowc) * p.Hq + h) * D + 32 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Qf[ks] = join(*(const u32x4*)(qp + 64 * ks), *(const u32x4*)(qp + 64 * ks + 16));
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
    ncol = c < ncol ? c : ncol;
  }

  // ---- tile copies: group 1 the K tiles, group 0 the V^T tiles, TPW per wavefront and vector phase
  // K tile: 64 rows (keys, clamped to the last one) of D bytes; V^T tile: D rows (always complete:
  // rows are padded to 64 keys in memory) of 64 bytes. Each copy instruction fills 1 KiB of LDS;
  // the swizzle is applied by choosing which global chunk a lane fetches.
  // (the per-lane byte offsets of an interior tile are computed once; a tile then costs one scalar
  // base address and TPW copy instructions. Only K tiles at the end of the sequence, whose rows have to
  // be clamped, recompute their addresses.)
  unsigned toff[TPW];
#pragma unroll
  for (int u = 0; u < TPW; ++u) {
    if (grp == 1) {
      const int r = ((w & 3) + 4 * u) * KRPI + lane / KCPR;
      toff[u] = (unsigned)(r * kstride + 16 * ((lane % KCPR) ^ swz_k8<KROWB>(r)));
    } else {
      const int r = ((w & 3) + 4 * u) * 16 + lane / 4;
      toff[u] = (unsigned)(r * a.vt_stride + 16 * ((lane % 4) ^ swz_v8(r)));
    }
  }
  auto issue_tile = [&](int j) {
    char* dst = smem + (j % RING) * BUFB;
    if (grp == 1) {
      if (j * BC + BC <= nk) {
        const char* base = (const char*)Kb + (long)j * BC * kstride;
#pragma unroll
        for (int u = 0; u < TPW; ++u) dma16_uniform(base, toff[u], dst + ((w & 3) + 4 * u) * KRPI * KROWB);
      } else {
        int ln = lane;
        asm volatile("" : "+v"(ln));  // (addresses of this rare path are not to be held in registers)
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
          const int rb = ((w & 3) + 4 * u) * KRPI;
          const int r = rb + ln / KCPR;
          const int c = (ln % KCPR) ^ swz_k8<KROWB>(r);
          int key = j * BC + r;
          key = key < nk - 1 ? key : nk - 1;
          dma16(Kb + (long)key * kstride + 16 * c, dst + rb * KROWB);
        }
      }
    } else {
      // (blocks past the end are requested like the others, their data is never read: stay inside the rows)
      const char* base = (const char*)Vb + (long)(j < ncol_all ? j : ncol_all - 1) * BC;
#pragma unroll
      for (int u = 0; u < TPW; ++u) dma16_uniform(base, toff[u], dst + KTILE + ((w & 3) + 4 * u) * 16 * 64);
    }
  };
  issue_tile(0);
  issue_tile(1);
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int t = 0; t < 8; ++t) touch(Qf[ks][t]);
  wait_vmem();
  lds_barrier();

  // ---- lane constants of the operand reads
  // K row of accumulator row lq = 8q + 4h' + u: key 16h' + 4q + u of the 32-key tile
  const int krow = 16 * ((lq >> 2) & 1) + 4 * (lq >> 3) + (lq & 3);
  const int kx = swz_k8<KROWB>(krow);            // (the same for both tiles: they are 32 rows apart)
  const int kbase = krow * KROWB;
  const int vx = swz_v8(lq);                      // (the same for every 32-row tile of V^T)
  const int vbase = KTILE + lq * 64;

  const float c2 = p.scale_log2e;  // scale * descale_q * descale_k * log2(e)
  const int wrow_last = prow0 + 31 + off;
  const int lim_row = CAUSAL ? (row + off < nk - 1 ? row + off : nk - 1) : nk - 1;

  f32x16 S[2];
  i32x8 Pf;

  // (the operands of both products come from LDS as they are needed; requesting them several MFMAs
  // early through a register ring, as the bf16 kernels do, measured 7% slower here)
  auto matrix_phase = [&](int j) {
    __builtin_amdgcn_s_setprio(2);
    if (j < ncol && (!CAUSAL || j * BC <= wrow_last)) {  // S^T = K_j Q_i^T (line 8)
      const char* kt_ = smem + (j % RING) * BUFB + kbase;
      S[0] = S[1] = (f32x16){0};
#pragma unroll
      for (int i = 0; i < 2 * KS; ++i) {
        const int kt = i & 1, ks = i >> 1, c0 = 4 * ks + 2 * hh;
        const char* rp = kt_ + 32 * kt * KROWB;
        const i32x8 x = join(*(const u32x4*)(rp + 16 * (c0 ^ kx)), *(const u32x4*)(rp + 16 * ((c0 + 1) ^ kx)));
        S[kt] = mfma_fp8(x, Qf[ks], S[kt]);
      }
    }
    if (j > 0 && (!CAUSAL || (j - 1) * BC <= wrow_last)) {  // O^T += V_{j-1}^T P^T (line 10)
      const char* vt_ = smem + ((j - 1) % RING) * BUFB + vbase;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const char* rp = vt_ + 32 * dt * 64;
        // keys 16 hh .. of tile 0, then of tile 1: the order of this lane half's exponentials
        const i32x8 x = join(*(const u32x4*)(rp + 16 * (hh ^ vx)), *(const u32x4*)(rp + 16 * ((2 + hh) ^ vx)));
        O[dt] = mfma_fp8(x, Pf, O[dt]);
      }
    }
    __builtin_amdgcn_s_setprio(0);
  };

  auto vector_phase = [&](int j) {  // online softmax of block j (line 9)
    if (j >= ncol || (CAUSAL && j * BC > wrow_last)) return;
    const int col0 = j * BC;
    const bool need_mask = (CAUSAL && col0 + BC - 1 > prow0 + off) || (col0 + BC > nk);
    if (need_mask) {
      asm volatile("; keep this a branch: the mask costs two instructions per element" ::);
      // register r of tile kt holds key col0 + 32 kt + 16 hh + r
      const int lim = lim_row - col0 - 16 * hh;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) S[kt][r] = 32 * kt + r > lim ? -INFINITY : S[kt][r];
    }
    float mx = fmaxf(S[0][0], S[1][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = __builtin_fmaxf(__builtin_fmaxf(mx, S[0][r]), S[1][r]);  // (one three-way maximum each)
    mx = max_with_partner32(mx);
    const float m_new = fmaxf(m, mx);
    // the operand format leaves no headroom above 2^8: the reference is the true running maximum
    // (column 0 is visible to every row and blocks are walked in ascending order: m_new is finite)
    if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {
      const float alpha = fast_exp2((m - m_new) * c2);
      l *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
      m = m_new;
    }
    const float mc = m * c2 - 8.f;  // exponentials times 2^8: the scaling of the operand, folded into the exponent
    float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; r += 4) {
        float e[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) e[u] = fast_exp2(__builtin_fmaf(S[kt][r + u], c2, -mc));
        rs0 += e[0] + e[2];
        rs1 += e[1] + e[3];
        // bytes 16 kt + r .. + 3 of this lane half's operand: P * 2^8 rounded to E4M3
        int word = 0;
        word = __builtin_amdgcn_cvt_pk_fp8_f32(e[0], e[1], word, false);
        word = __builtin_amdgcn_cvt_pk_fp8_f32(e[2], e[3], word, true);
        Pf[4 * kt + r / 4] = word;
      }
    l += rs0 + rs1;  // (in units of 2^-8)
  };

  // phases: see fwd_kernel (both barriers of a block are kept here: leaving out the one that follows
  // no wait, as the bf16 kernels with one workgroup per compute unit do, measured 1-4% slower; the
  // vector phase is the longer one in this kernel)
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

  // ---- epilogue: O = diag(l)^-1 O * descale_v, L = m + log l (lines 12-15); l and O both carry
  //      the factor 2^8 of the operand scaling, which cancels in O and is taken out of L
  const float lsum = sum_with_partner32(l);
  const float inv = a.descale_v / lsum;
  wait_vmem();    // the copies issued past the last block have landed:
  lds_barrier();  // the ring is free for staging the output rows
  {
    // 32 columns of the head dimension at a time (32 rows of 32 bf16 per wavefront)
    char* stg = smem + w * 2048;
    static_assert(RING * BUFB >= 8 * 2048, "the ring holds every wavefront's staging area");
    __bf16* op = a.O + (((long)s * n + prow0) * p.Hq + h) * D;
    const long ostride = (long)p.Hq * D;
    int ln = lane;
    asm volatile("" : "+v"(ln));
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) store_rows_via_lds<1, false>(stg, &O[dt], inv, op + 32 * dt, ostride, n - prow0, 32, ln);
    if (row < n && hh == 0)
      a.LSE[s * p.lse_seq_stride + h * p.lse_head_stride + row] = m * p.scale + (fast_log2(lsum) - 8.f) * kLn2;
  }
}

hipError_t launch_fwd_fp8(const Fp8Args& a, int d, int causal, hipStream_t st) {
  dim3 grid(grid_size((a.p.N + 255) / 256, a.p.Hq * a.p.nseq)), block(512);
  if (d == 128) {
    if (causal) hipLaunchKernelGGL((fwd_fp8_kernel<128, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((fwd_fp8_kernel<128, false>), grid, block, 0, st, a);
  } else {
    if (causal) hipLaunchKernelGGL((fwd_fp8_kernel<64, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((fwd_fp8_kernel<64, false>), grid, block, 0, st, a);
  }
  return hipGetLastError();
}

}  // namespace fa
