// Shared device-side helpers for the gfx950 attention kernels: vector types,
// MFMA wrappers and the lane layouts they imply.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Problem description shared by the forward and backward kernels. A "sequence"
// is one batch entry (dense) or one entry of cu_seqlens (packed ragged). A sequence has
// nq query rows and nk key/value rows (equal except through the two-length entry points);
// under the causal mask query r stands at position r + nk - nq of the keys.
struct Problem {
  const int32_t* cu_seqlens;  // device, nseq + 1 entries; nullptr for the dense layout
  const int32_t* cu_seqlens_k;  // ragged with two lengths: the key/value rows' offsets; else nullptr
  int nseq;                   // number of sequences (dense: batch size)
  int N;                      // dense: number of query rows; ragged: upper bound on any length
  int Nk;                     // dense: number of key/value rows; ragged: same bound
  int Hq, Hkv, G;             // G = Hq / Hkv
  int d;                      // head dimension in memory (a multiple of 8); kernels pad it to 64 or 128 on chip
  int total_tokens;
  long lse_seq_stride;        // dense: Hq * N, ragged: 0
  long lse_head_stride;       // dense: N, ragged: total_tokens
  float scale;                // softmax scaling
  float scale_log2e;          // scale * log2(e)
  int f16;                    // element type of the 16-bit tensors: 0 bfloat16, 1 IEEE half precision
  // dropout on P (drop_thr = 0: none): an entry is kept when its byte of the hash is >= drop_thr
  uint32_t drop_thr;          // round(256 p), 1 .. 255
  uint32_t drop_seed;         // (seed mod 2^32) xor (seed >> 32) * 0x27D4EB2F
  float drop_rp;              // 1 / (1 - drop_thr / 256)
  // elementwise mask added to the scaled scores (nullptr: none): bfloat16, finite or -inf,
  // element (s, h, r, c) at mask[s * mask_bs + h * mask_hs + r * mask_rs + c]; a stride of 0
  // shares the mask over sequences or heads; mask_rs >= Nk rounded up to 8, a multiple of 8
  const __bf16* mask;
  long mask_bs, mask_hs, mask_rs;
  // sliding window (local attention): with query r at position q = r + nk - nq among the keys, key c
  // is visible iff q - win_left <= c <= q + win_right; a negative bound is no bound. Only read
  // by the LOCAL instantiations (the entry points send "no bound at all" and "win_right = 0
  // alone" to the plain and the causal kernels).
  int win_left, win_right;
  // block-sparse pattern (nullptr: none; LOCAL instantiations only): one byte per block of
  // 2^bmask_log2 x 2^bmask_log2 entries of S (a power of two, at least 64), row blocks counted
  // from query 0 and key blocks from key 0; byte (s, h, rb, cb) at
  // bmask[s * bmask_bs + h * bmask_hs + rb * bmask_cols + cb], 0 = the block is removed;
  // a stride of 0 shares the pattern over sequences or heads
  const uint8_t* bmask;
  long bmask_bs, bmask_hs;
  int bmask_cols, bmask_log2;
};
constexpr int kPatternWords = 64;  // 64-bit words of a wavefront's activity bitmap in LDS: 4096 blocks or tiles

struct SeqInfo {
  long tok0;   // first query row of the sequence in the packed [tokens, H, d] view
  long tok0k;  // first key/value row
  int n;       // query rows
  int nk;      // key/value rows
};

__device__ __forceinline__ SeqInfo seq_info(const Problem& p, int s) {
  SeqInfo r;
  if (p.cu_seqlens) {
    int a = p.cu_seqlens[s];
    r.tok0 = r.tok0k = a;
    r.n = r.nk = p.cu_seqlens[s + 1] - a;
    if (p.cu_seqlens_k) {
      a = p.cu_seqlens_k[s];
      r.tok0k = a;
      r.nk = p.cu_seqlens_k[s + 1] - a;
    }
  } else {
    r.tok0 = (long)s * p.N;
    r.tok0k = (long)s * p.Nk;
    r.n = p.N;
    r.nk = p.Nk;
  }
  return r;
}

// Launch index -> (block of rows or columns, head, sequence).
//
// The chip has 8 XCDs, each with 32 CUs and a private 4 MiB L2; the hardware hands
// consecutive workgroup indices to consecutive XCDs. Every workgroup of one (head,
// sequence) pair streams the same K/V (or Q/dO) through L2, about 4 MiB at d = 128 and
// N = 8192. The mapping below therefore gives all blocks of a pair to ONE XCD and lets an
// XCD walk its pairs one after the other, so its 32 CUs share one pair's operands at a time
// instead of thrashing L2 with eight. Under the causal mask block costs differ by up to
// the number of blocks, so there the XCD's pairs are interleaved and all their heaviest
// blocks are dispatched first (longest-processing-time order), lightest last. Kernels are launched on grid_size(nblk, pairs) workgroups; indices that
// fall past the last pair return valid = false.
constexpr int kXcds = 8;
struct BlockCoord {
  int blk, head, seq;
  bool valid;
};
__host__ __device__ inline unsigned grid_size(int nblk, int pairs) {
  return (unsigned)(((pairs + kXcds - 1) / kXcds) * kXcds * nblk);
}
// `group` > 1 (kernels whose grid runs over QUERY heads that share key/value heads in groups of
// that size): heads are handed out so that the heads of one group follow each other at a
// distance of nheads / group pairs. With a multiple of 8 key/value heads they then land on the
// same XCD, whose L2 holds the group's K and V once instead of every XCD holding them all.
template <bool WORK_SORTED>
__device__ __forceinline__ BlockCoord block_coord(int nblk, int nheads, int nseq, int group = 1) {
  const int L = blockIdx.x;
  const int x = L % kXcds, k = L / kXcds;
  const int ppx = gridDim.x / (kXcds * nblk);  // pairs per XCD
  int pl;                                       // which of this XCD's pairs
  BlockCoord c;
  if (WORK_SORTED) {  // causal: the XCD's pairs take turns, every pair's heaviest blocks first
    c.blk = k / ppx;
    pl = k % ppx;
  } else {  // one pair at a time
    c.blk = k % nblk;
    pl = k / nblk;
  }
  const int pr = pl * kXcds + x;
  const int hp = pr % nheads, nkv = nheads / group;
  c.head = (hp % nkv) * group + hp / nkv;
  c.seq = pr / nheads;
  c.valid = pr < nheads * nseq;
  return c;
}

// D = A(32 x 16) * B(16 x 32) + C on one wavefront, 16-bit inputs, fp32 accumulate.
// Lane l supplies A[l % 32][8 * (l / 32) + t] and B[8 * (l / 32) + t][l % 32], t = 0..7,
// and owns C[8 * (r / 4) + 4 * (l / 32) + (r % 4)][l % 32] in register r = 0..15.
// The kernels move 16-bit elements around as raw bits (bf16x8 is just 128 bits of them);
// the element type only matters here, where they are multiplied, and in pack2 below, where
// float32 results are rounded: F16 = false means bfloat16, F16 = true IEEE half precision.
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
template <bool F16 = false>
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of the 32 x 32 accumulator tile that register r of lane-half hh holds.
__device__ __forceinline__ constexpr int acc_row(int r, int hh) { return 8 * (r / 4) + 4 * hh + (r % 4); }

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Transposing LDS read (ds_read_b64_tr_b16). Within each group of 16 lanes,
// lane p passes the address of 4 consecutive 16-bit elements; lane i receives,
// in slot t, element (i % 4) of the four that lane (i / 4 + 4 * t) pointed at.
__device__ __forceinline__ s16x4 lds_read_tr(const __bf16* ptr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)ptr);
}

// Maximum / sum of a value with the one held by lane l ^ 32 (v_permlane32_swap).
__device__ __forceinline__ float max_with_partner32(float x) {
  int xi = __builtin_bit_cast(int, x);
  auto sw = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return fmaxf(__builtin_bit_cast(float, (int)sw[0]), __builtin_bit_cast(float, (int)sw[1]));
}

__device__ __forceinline__ float sum_with_partner32(float x) {
  int xi = __builtin_bit_cast(int, x);
  auto sw = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return __builtin_bit_cast(float, (int)sw[0]) + __builtin_bit_cast(float, (int)sw[1]);
}

// Two float32 values rounded (to nearest even) to the 16-bit element type, packed low | high.
template <bool F16 = false>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  f32x2 v = {lo, hi};
  if constexpr (F16) {
    f16x2 r = __builtin_convertvector(v, f16x2);
    return __builtin_bit_cast(uint32_t, r);
  } else {
    bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
  }
}

// Registers 8s .. 8s+7 of an accumulator tile, rounded to the element type, as an MFMA operand.
template <bool F16 = false>
__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int s) {
  u32x4 r;
  r[0] = pack2<F16>(v[8 * s + 0], v[8 * s + 1]);
  r[1] = pack2<F16>(v[8 * s + 2], v[8 * s + 3]);
  r[2] = pack2<F16>(v[8 * s + 4], v[8 * s + 5]);
  r[3] = pack2<F16>(v[8 * s + 6], v[8 * s + 7]);
  return __builtin_bit_cast(bf16x8, r);
}

// Element t of 8 raw 16-bit elements, widened to float32.
template <bool F16>
__device__ __forceinline__ float widen(bf16x8 v, int t) {
  if constexpr (F16) return (float)__builtin_bit_cast(f16x8, v)[t];
  else return (float)v[t];
}

// The 16-bit element in the low (hi = false) or high half of a 32-bit word, widened to float32.
template <bool F16>
__device__ __forceinline__ float widen_half(uint32_t w, bool hi) {
  if constexpr (F16) return (float)__builtin_bit_cast(_Float16, (unsigned short)(hi ? w >> 16 : w));
  else return __builtin_bit_cast(float, hi ? (w & 0xffff0000u) : (w << 16));
}

// Dropout generator (defined by this library, the same function as the CPU checker's): for
// head index bh = sequence * Hq + head, query r and key c,
//   x = (c / 4) * 0x9E3779B1 + r * 0x85EBCA77 + (seed_mix xor bh * 0xC2B2AE3D), mixed by
//   drop_mix; entry (r, c) is kept when byte c % 4 of x is >= the threshold.
constexpr uint32_t kDropCol = 0x9E3779B1u, kDropRow = 0x85EBCA77u, kDropHead = 0xC2B2AE3Du;
__device__ __forceinline__ uint32_t drop_mix(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  x *= 0x846CA68Bu;
  x ^= x >> 16;
  return x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

}  // namespace fa
