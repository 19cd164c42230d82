// LDS machinery shared by the forward and backward kernels: swizzled tiles,
// direct global -> LDS tile loads, operand reads and the LDS-only barrier.
#pragma once
#include "fa_common.h"

namespace fa {

// Workgroup barrier that only waits for this wavefront's LDS traffic: global
// loads and atomics that are still in flight stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// Wait until at most N of this wavefront's global loads (they complete in order) are outstanding.
template <int N>
__device__ __forceinline__ void wait_vmem_upto() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// ---- swizzled LDS tiles -----------------------------------------------------
// Tiles are stored without padding, rows of ROWB = 128 or 256 bytes, as 16-byte
// chunks whose position inside the row is XOR-ed with a function of the row. The
// function is chosen so that BOTH access patterns used here are conflict free:
//   * 16-byte row reads, 16 consecutive rows at the same chunk index, and
//   * transposing 8-byte reads, 4 consecutive rows x 64 contiguous bytes.
template <int ROWB>
__device__ __forceinline__ int swz(int row) {
  if (ROWB == 256) return ((row & 3) << 2) | ((row >> 2) & 3);
  const int k = (row >> 1) & 7;  // two 128-byte rows share one 256-byte bank line
  return ((k & 1) << 2) | (k >> 1);
}
template <int ROWB>
__device__ __forceinline__ int swz_off(int row, int chunk) { return row * ROWB + 16 * (chunk ^ swz<ROWB>(row)); }

// 16 bytes per lane from global memory straight into LDS (global_load_lds_dwordx4): lane i's
// data lands at lds + 16 * i, `lds` being wave-uniform. Written as inline assembly on
// purpose: the compiler would otherwise make every later LDS read wait for ALL outstanding
// copies (it cannot tell the ring buffers apart), which serialises the prefetch. The
// kernels order these copies themselves with wait_vmem*() + barriers. M0 holds the LDS
// base for the duration of the instruction only; the compiler keeps no value live in M0.
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const char*)p;
}
__device__ __forceinline__ void dma16(const void* gaddr, const void* lds) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gaddr),
               "s"(__builtin_amdgcn_readfirstlane(lds_address(lds)))
               : "memory");
}
// same with a wave-uniform base pointer and a 32-bit per-lane byte offset
__device__ __forceinline__ void dma16_uniform(const void* gbase, unsigned voff, const void* lds) {
  // the base must sit in scalar registers whatever the compiler believes about its uniformity
  const unsigned long long b = (unsigned long long)gbase;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)b), hi = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32));
  gbase = (const void*)(((unsigned long long)hi << 32) | lo);
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(gbase),
               "s"(__builtin_amdgcn_readfirstlane(lds_address(lds)))
               : "memory");
}

// Copy `nrows` rows of D bf16 elements (row pitch `gstride` elements, first row
// `row_first`, rows clamped to `row_last`) from global memory straight into a
// swizzled LDS tile, 16 bytes per lane, without passing through registers. Each
// wavefront instruction fills 1 KiB of consecutive LDS; the swizzle is applied by
// choosing which global chunk each lane fetches.
//
// PAD: the rows in memory hold only `nchunk` < D / 8 chunks (a head dimension below the
// tile width D). Lanes whose chunk lies past the row end copy nothing; the kernel zeroes
// the whole LDS block once before its first copy, and because a given LDS position always
// receives the same chunk index those positions stay zero for every later tile.
template <int D, int NROWS, int NW, bool PAD = false>
__device__ __forceinline__ void tile_load_async(char* tile, const __bf16* gbase, long gstride, int row_first,
                                                int row_last, int wave, int lane, int nchunk = D / 8) {
  constexpr int ROWB = 2 * D, CPR = ROWB / 16, RPI = 64 / CPR, NI = NROWS / RPI;
  static_assert(NI % NW == 0, "tile must divide over the wavefronts");
  // The lane index is hidden from the optimiser: this is the rarely taken path of the streaming
  // kernels (tiles at the end of a sequence), and otherwise the loop-invariant parts of its
  // per-lane 64-bit addresses are kept in registers across the whole main loop.
  asm volatile("" : "+v"(lane));
#pragma unroll
  for (int u = 0; u < NI / NW; ++u) {
    const int rb = (wave + NW * u) * RPI;
    const int r = rb + lane / CPR;
    const int c = (lane % CPR) ^ swz<ROWB>(r);
    int grow = row_first + r;
    grow = grow < row_last ? grow : row_last;
    if (!PAD || c < nchunk) dma16(gbase + (long)grow * gstride + 8 * c, tile + rb * ROWB);
  }
}

// Zero an LDS block (all threads of the workgroup), then a barrier: PAD kernels call this
// before their first copy.
template <int NTHREADS>
__device__ __forceinline__ void lds_zero(char* smem, int bytes) {
  for (int i = threadIdx.x * 16; i < bytes; i += NTHREADS * 16) *(u32x4*)(smem + i) = (u32x4){0, 0, 0, 0};
  __syncthreads();
}

__device__ __forceinline__ bf16x8 lds_b128(const char* smem, int off) { return *(const bf16x8*)(smem + off); }
__device__ __forceinline__ bf16x8 lds_tr_pair(const char* smem, int off_lo, int off_hi) {
  s16x4 lo = lds_read_tr((const __bf16*)(smem + off_lo));
  s16x4 hi = lds_read_tr((const __bf16*)(smem + off_hi));
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}
// The same copy for kernels that stream many tiles of one tensor: the per-lane byte offsets
// of an interior tile are computed once (TileLoader::init) and every tile then costs one
// scalar base-address update plus the load instructions. Tiles that reach past `row_last`
// take the clamping path above.
template <int D, int NROWS, int NW, bool PAD = false>
struct TileLoader {
  static constexpr int ROWB = 2 * D, CPR = ROWB / 16, RPI = 64 / CPR, NI = NROWS / RPI, PER = NI / NW;
  static_assert(NI % NW == 0, "tile must divide over the wavefronts");
  unsigned voff[PER];  // byte offset of this lane's chunk from the tile's first row
  unsigned on;         // PAD: bit u set when copy u of this lane fetches a chunk that exists
  int nchunk;
  __device__ __forceinline__ void init(long gstride, int wave, int lane, int nchunk_ = D / 8) {
    on = 0;
    nchunk = nchunk_;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int r = (wave + NW * u) * RPI + lane / CPR;
      const int c = (lane % CPR) ^ swz<ROWB>(r);
      voff[u] = (unsigned)(r * gstride + 8 * c) * 2u;
      if (c < nchunk_) on |= 1u << u;
    }
  }
  // an interior tile whose first row starts at `first_row` (wave-uniform)
  __device__ __forceinline__ void load_at(char* tile, const __bf16* first_row, int wave) const {
#pragma unroll
    for (int u = 0; u < PER; ++u)
      if (!PAD || ((on >> u) & 1)) dma16_uniform(first_row, voff[u], tile + (wave + NW * u) * RPI * ROWB);
  }
  __device__ __forceinline__ void load(char* tile, const __bf16* gbase, long gstride, int row_first, int row_last,
                                       int wave, int lane) const {
    if (row_first + NROWS - 1 <= row_last) {
      const char* base = (const char*)(gbase + (long)row_first * gstride);  // wave-uniform
#pragma unroll
      for (int u = 0; u < PER; ++u)
        if (!PAD || ((on >> u) & 1)) dma16_uniform(base, voff[u], tile + (wave + NW * u) * RPI * ROWB);
    } else {
      tile_load_async<D, NROWS, NW, PAD>(tile, gbase, gstride, row_first, row_last, wave, lane, nchunk);
    }
  }
};

// Tell the compiler that a value loaded from global memory is needed NOW. The kernels
// order their direct-to-LDS copies with hand-written s_waitcnt (the compiler does not see
// those copies), so the compiler never learns that ordinary loads issued before the main
// loop have long completed and would re-wait for them, with vmcnt(0), inside the loop,
// which also waits for every copy in flight. Touching the values once before the loop makes
// it place that wait there.
template <class T>
__device__ __forceinline__ void touch(const T& x) {
  asm volatile("" ::"v"(x));
}

// 16 bytes per lane from global memory into registers, hidden from the compiler's own
// bookkeeping of loads in flight (it would wait for them with vmcnt(0), which also waits for
// every direct-to-LDS copy in flight). The value may only be used after a hand-written wait
// that covers the load, and only through landed(), which pins the first use behind that wait.
// (dst is declared read-write so that the new value takes the old one's registers: reloading a
// long-lived operand in place then costs neither registers nor copies.)
template <int OFF>
__device__ __forceinline__ void load16_async(u32x4& dst, const void* gaddr) {
  asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "+v"(dst) : "v"(gaddr), "n"(OFF) : "memory");
}
template <class T>
__device__ __forceinline__ void landed(T& x) {
  asm volatile("; landed %0" : "+v"(x));  // (the comment lets a checker of the compiler's output find this place)
}

// Write a wavefront's 32 rows x (32 NT) columns, held TRANSPOSED in accumulators (register r of
// tile t in lane (lq, hh) is row lq, column 32 t + acc_row(r, hh)), to global memory as
// 16-bit rows, scaled by the lane's row factor `mul`. Storing straight from that layout puts 16
// bytes per row into every instruction (32 partly written cache lines each); going through a
// wavefront-private LDS buffer `stg` (32 * 64 * NT bytes, chunks XOR-ed so that neither side
// conflicts) turns it into whole rows: a quarter of the write requests. Rows >= nrows and columns >=
// ncols (a multiple of 8) are not stored. Needs no barrier: only this wavefront touches `stg`.
template <int NT, bool F16>
__device__ __forceinline__ void store_rows_via_lds(char* stg, const f32x16* acc, float mul, __bf16* g, long gstride,
                                                   int nrows, int ncols, int lane) {
  constexpr int SROW = 64 * NT;      // bytes per staged row
  constexpr int CPR = SROW / 16;     // 16-byte chunks per row
  constexpr int RPB = 256 / SROW;    // rows per 256 bytes (one pass over the banks)
  constexpr int RPI = 64 / CPR;      // rows per store instruction
  const int lq = lane & 31, hh = lane >> 5;
  char* wr = stg + lq * SROW + 8 * hh;
  const int wx = (lq / RPB) & (CPR - 1);
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      u32x2 o;
      o[0] = pack2<F16>(acc[t][4 * r4 + 0] * mul, acc[t][4 * r4 + 1] * mul);
      o[1] = pack2<F16>(acc[t][4 * r4 + 2] * mul, acc[t][4 * r4 + 3] * mul);
      *(u32x2*)(wr + 16 * ((4 * t + r4) ^ wx)) = o;
    }
  const int c = lane % CPR, rr = lane / CPR;
#pragma unroll
  for (int u = 0; u < 32 / RPI; ++u) {
    const int row = RPI * u + rr;
    const u32x4 v = *(const u32x4*)(stg + row * SROW + 16 * (c ^ ((row / RPB) & (CPR - 1))));
    if (row < nrows && 8 * c < ncols) *(u32x4*)(g + row * gstride + 8 * c) = v;
  }
}

// The same for NT tiles where NT need not be a power of two (three tiles: one at a time).
template <int NT, bool F16>
__device__ __forceinline__ void store_tiles_via_lds(char* stg, const f32x16* acc, float mul, __bf16* g, long gstride,
                                                    int nrows, int ncols, int lane) {
  if constexpr ((NT & (NT - 1)) == 0) {
    store_rows_via_lds<NT, F16>(stg, acc, mul, g, gstride, nrows, ncols, lane);
  } else {
#pragma unroll
    for (int t = 0; t < NT; ++t) store_rows_via_lds<1, F16>(stg, acc + t, mul, g + 32 * t, gstride, nrows, ncols - 32 * t, lane);
  }
}

// Issue-order hints for the machine scheduler (one scheduling group each, in program
// order): without them the compiler tends to wait for every LDS operand right before
// the MFMA that uses it, which exposes the LDS latency once per MFMA.
#define FA_SCHED_MFMA(n) __builtin_amdgcn_sched_group_barrier(0x008, n, 0)
#define FA_SCHED_DSRD(n) __builtin_amdgcn_sched_group_barrier(0x100, n, 0)

struct OperandPair {
  bf16x8 a, b;
};

// A sequence of N MFMAs whose operands come from LDS, with the operand reads issued
// AHEAD MFMAs early. load(i) returns the operand(s) of MFMA i (a bf16x8 or an
// OperandPair), mma(i, operands) performs MFMA i; READS is the number of LDS read
// instructions load(i) takes. The two halves can be called apart when the first reads may
// start earlier than the MFMAs (before a barrier, say): begin() issues the reads of MFMAs
// 0 .. AHEAD-1 into `ring`, run() does everything else.
template <int N, int AHEAD, int READS, class T, class LoadF>
__device__ __forceinline__ void mfma_stream_begin(T (&ring)[AHEAD], LoadF load) {
#pragma unroll
  for (int i = 0; i < AHEAD && i < N; ++i) ring[i] = load(i);
  FA_SCHED_DSRD(READS * (AHEAD < N ? AHEAD : N));
}
template <int N, int AHEAD, int READS, class T, class LoadF, class MmaF>
__device__ __forceinline__ void mfma_stream_run(T (&ring)[AHEAD], LoadF load, MmaF mma) {
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const T cur = ring[i % AHEAD];
    if (i + AHEAD < N) {
      ring[i % AHEAD] = load(i + AHEAD);
      FA_SCHED_DSRD(READS);
    }
    mma(i, cur);
    FA_SCHED_MFMA(1);
  }
}
template <int N, int AHEAD, int READS, class LoadF, class MmaF>
__device__ __forceinline__ void mfma_stream(LoadF load, MmaF mma) {
  decltype(load(0)) ring[AHEAD];
  mfma_stream_begin<N, AHEAD, READS>(ring, load);
  mfma_stream_run<N, AHEAD, READS>(ring, load, mma);
}

}  // namespace fa
