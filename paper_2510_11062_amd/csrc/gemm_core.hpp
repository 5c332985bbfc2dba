// Workgroup-tile contraction on the gfx950 matrix cores.
//
// One workgroup produces a 256 x 256 fp32 tile
//   C[a, b] = sum_k A[a, k] * B[b, k]
// from two operands that are both contiguous along k ("NT" layout; a second entry point takes both
// operands k-major).  Its wavefronts share the tile as a WaveGrid (below): 8 wavefronts of 64 x 128
// (2 x 4 MFMA 32x32 accumulator blocks, 128 accumulator registers per lane) or 4 wavefronts of 128 x 128
// (4 x 4 blocks, 256 registers).  k is consumed in steps of 128 bytes per row (64 bf16 or 32 fp32 elements).
//
// Data path: global -> LDS with direct-to-LDS loads (global_load_lds_dwordx4, 16 bytes per lane,
// one instruction fills 8 rows x 128 bytes) into a ring of five 32 KiB slots (one operand panel each);
// LDS -> registers with ds_read_b128, fragments fetched one 16-wide sub-step ahead of the MFMAs that
// consume them.  The 16-byte chunk index of every row is XOR-swizzled (applied on the global side of the
// direct loads, since their LDS side is fixed to lane * 16) so that the fragment reads are free of bank
// conflicts.  The direct loads are issued through inline asm: the compiler would otherwise make every
// later LDS read wait for all outstanding direct loads.  Their completion is enforced by hand with
// s_waitcnt vmcnt in front of the one workgroup barrier per k-step.
//
// Instruction order: a wavefront that issues a burst of LDS reads or direct loads keeps its SIMD's
// matrix pipe idle for the length of the burst (wavefronts that share a SIMD run in step, so the other
// one rarely fills the gap).  The loop body is therefore written out as a fixed sequence, pinned with
// scheduling barriers, in which every MFMA is followed by at most one LDS read and one direct load:
// each memory instruction issues in the shadow of an MFMA that is already executing.  When which panel
// is requested is described at pinned_k_step.
//
// Accumulator layout (per lane, block (i, j), register r = 0..15; 8-wavefront grid):
//   a = wm*64 + i*32 + 8*(r/4) + 4*(lane/32) + (r%4)        (A row inside the tile)
//   b = wn*128 + j*32 + lane%32                              (B row inside the tile)
#pragma once

#include "common.hpp"

namespace atg {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int kTile = 256;                       // rows of each operand per tile
constexpr int kStepBytes = 128;                  // bytes of k per row per step
constexpr int kLdsOperand = kTile * kStepBytes;  // 32 KiB

// How the wavefronts of a workgroup share the 256 x 256 tile: WA x WB wavefronts, each owning a
// (256 / WA) x (256 / WB) sub-tile.  Two layouts are used:
//   WaveGrid<4, 2>  8 wavefronts, two per SIMD, 64 x 128 each (128 accumulator registers): the second
//                   wavefront of a SIMD covers part of the other's per-tile prologue and epilogue, which
//                   matters when the k loop is short (forward kernels: k = H);
//   WaveGrid<2, 2>  4 wavefronts, one per SIMD, 128 x 128 each (256 accumulator registers): a third fewer
//                   LDS fragment reads per MFMA and half as many wavefronts at each barrier; faster once
//                   the k loop is long and the epilogue light (dHidden: k = V); slower on short loops, and
//                   slower for dW, whose epilogue adds 256 fp32 values per lane to memory.
template <int WA, int WB>
struct WaveGrid {
  static constexpr int kWavesA = WA, kWavesB = WB;
  static constexpr int kThreads = WA * WB * 64;
  static constexpr int kIB = kTile / WA / 32;              // accumulator block rows per wavefront
  static constexpr int kJB = kTile / WB / 32;              // accumulator block columns per wavefront
  static constexpr int kRowsPerWave = kTile / (WA * WB);   // operand rows each wavefront loads
  static constexpr int kLoadsPerWave = kRowsPerWave / 8;   // direct-load instructions per operand
  static constexpr int kMmPerSub = kIB * kJB;              // MFMA groups per 16-wide sub-step
  static constexpr int kRdPerSub = kIB + kJB;              // fragment reads per sub-step
  static constexpr int kRdEvery = kMmPerSub / kRdPerSub;   // a fragment read follows every kRdEvery-th MFMA
};
using G8 = WaveGrid<4, 2>;
using G4 = WaveGrid<2, 2>;

// the 8-wavefront layout under its short names (forward, exponentials, dZ)
constexpr int kWavesA = G8::kWavesA, kWavesB = G8::kWavesB;
constexpr int kGemmThreads = G8::kThreads;
constexpr int kIB = G8::kIB, kJB = G8::kJB;

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

template <typename T>
struct Mma;

template <>
struct Mma<bf16_t> {
  // one v_mfma_f32_32x32x16_bf16: each lane supplies 8 consecutive k of its row
  static __device__ __forceinline__ void run(const uint4& a, const uint4& b, floatx16& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};

template <>
struct Mma<float> {
  // four v_mfma_f32_32x32x2_f32: each lane supplies 4 consecutive k of its row
  static __device__ __forceinline__ void run(const uint4& a, const uint4& b, floatx16& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
  }
};

template <typename G>
struct TileCoordT {
  int lane, wm, wn, half;
  __device__ __forceinline__ TileCoordT() {
    lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    wm = wave / G::kWavesB;
    wn = wave % G::kWavesB;
    half = lane >> 5;
  }
  // A row (inside the tile) of accumulator register r of block row i
  __device__ __forceinline__ int a_row(int i, int r) const {
    return wm * (kTile / G::kWavesA) + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
  }
  // B row (inside the tile) of block column j
  __device__ __forceinline__ int b_row(int j) const { return wn * (kTile / G::kWavesB) + j * 32 + (lane & 31); }
};
using TileCoord = TileCoordT<G8>;

// 16 bytes per lane, global -> LDS at (wave-uniform) lds_addr + lane * 16.
__device__ __forceinline__ void direct_load16(const char* g, uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(g), "s"(lds_addr_uniform)
               : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const char* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (__attribute__((address_space(3))) const char*)p));
}

// Workgroup barrier that orders LDS traffic only: waits for this wavefront's LDS operations
// (lgkmcnt(0)), not for its outstanding global stores.  __syncthreads() would also wait until every
// store issued so far has been acknowledged by memory, which an epilogue that has just written its
// results does not need before the LDS buffer is reused.
__device__ __forceinline__ void barrier_lds_only() {
  __builtin_amdgcn_s_waitcnt(0xC07F);   // vmcnt and expcnt at their maxima, lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
}

// Pinned k loop shared by both operand layouts.  Ops supplies
//   G                         the WaveGrid
//   mm(f, n)                  MFMA group n (0..kIB*kJB-1) on fragment set f
//   rd(sa, sb, ks, f, n)      fetch of fragment n (0..kIB+kJB-1) of sub-step ks into set f; sa / sb are the
//                             LDS byte offsets of the slots that hold the step's A and B panels
//   ld_a(slot, q), ld_b(slot, q)   direct load q (0..kLoadsPerWave-1) of the next A / B panel not yet
//                             requested, into the slot at LDS byte offset `slot`
//
// LDS is a ring of five 32 KiB slots, one operand panel (256 rows x 128 bytes) each: the A and B panels of
// k-step kt sit in slots (2 kt) % 5 and (2 kt + 1) % 5.  While step kt is consumed, the three other slots
// receive B of step kt+1 and A of step kt+2 (and may still be receiving A of step kt+1): up to 96 KiB of
// loads are in flight per compute unit, and every load has at least three sub-steps (of four per k-step) to
// land.  (Two 64 KiB stages, the obvious layout, leave the last loads of a step one sub-step: the loop then
// waits for memory at every barrier; with the loads removed altogether the same instruction sequence runs
// at 1.6 PFLOP/s, with two stages at 1.26-1.30.)  Per k-step:
//   sub-steps 0, 1   request A of step kt+2 (half the loads each), into the slot B of step kt-1 left
//   sub-step 2       no requests
//   wait until all but those A loads have landed; workgroup barrier (one per k-step)
//   sub-step 3       request B of step kt+2 into the slot A of step kt has just left; fetch the first
//                    fragments of step kt+1
// The loop guarantees: panels are requested in order of k; a slot is only overwritten after the barrier
// that follows its last read; a workgroup barrier separates the last LDS read from the return, so the
// caller may reuse the whole buffer at once.
constexpr int kLdsSlots = 5;
constexpr int kLdsSlot = kLdsOperand;              // 32 KiB
constexpr int kLdsBytes = kLdsSlots * kLdsSlot;    // 160 KiB: all of a compute unit's LDS

// index of the MFMA after which load k of `cnt` is issued within one sub-step: evenly spread, so
// that the wavefronts of the workgroup do not queue up behind each other at the load unit
__device__ __forceinline__ constexpr int load_slot(int k, int cnt, int mm_per_sub) {
  return ((2 * k + 1) * mm_per_sub) / (2 * cnt);
}

#define ATG_PIN() __builtin_amdgcn_sched_barrier(0)

// s_waitcnt vmcnt(N) with expcnt and lgkmcnt left at their maxima (N < 64)
template <int N>
__device__ __forceinline__ void wait_direct_loads_but() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 0xF) | ((N >> 4) << 14));
}

__device__ __forceinline__ int ring_slot(int first, int i) {
  int s = first + i;
  if (s >= kLdsSlots) s -= kLdsSlots;
  return s * kLdsSlot;
}

// One k-step.  `first` = (2 kt) % 5.  HAS_NEXT: step kt+1 exists (its first fragments are fetched);
// HAS_NEXT2: step kt+2 exists (its panels are requested).
template <bool HAS_NEXT, bool HAS_NEXT2, typename Ops>
__device__ __forceinline__ void pinned_k_step(Ops& ops, int first) {
  using G = typename Ops::G;
  constexpr int kMmPerSub = G::kMmPerSub, kRdPerSub = G::kRdPerSub, kRdEvery = G::kRdEvery;
  constexpr int kLd = G::kLoadsPerWave, kHalf = kLd / 2;
  const int sa = ring_slot(first, 0), sb = ring_slot(first, 1);           // this step
  const int na = ring_slot(first, 2), nb = ring_slot(first, 3);           // step kt+1
  const int la = ring_slot(first, 4), lb = sa;                            // where step kt+2 goes
#pragma unroll
  for (int ss = 0; ss < 3; ++ss) {
    const int f = ss & 1;
#pragma unroll
    for (int n = 0; n < kMmPerSub; ++n) {
      ops.mm(f, n);
      ATG_PIN();
      if (n % kRdEvery == 0 && n / kRdEvery < kRdPerSub) {
        ops.rd(sa, sb, ss + 1, f ^ 1, n / kRdEvery);
        ATG_PIN();
      }
      if (HAS_NEXT2 && ss < 2) {
#pragma unroll
        for (int k = 0; k < kHalf; ++k)
          if (load_slot(k, kHalf, kMmPerSub) == n) {
            ops.ld_a(la, ss * kHalf + k);
            ATG_PIN();
          }
      }
    }
  }
  // everything but the A panel requested above has landed for this wavefront ...
  if (HAS_NEXT2) wait_direct_loads_but<kLd>();
  else wait_direct_loads_but<0>();
  __syncthreads();       // ... and for everyone, and everyone holds its last fragments of this step
  ATG_PIN();
#pragma unroll
  for (int n = 0; n < kMmPerSub; ++n) {
    ops.mm(1, n);
    ATG_PIN();
    if (HAS_NEXT && n % kRdEvery == 0 && n / kRdEvery < kRdPerSub) {
      ops.rd(na, nb, 0, 0, n / kRdEvery);
      ATG_PIN();
    }
    if (HAS_NEXT2) {
#pragma unroll
      for (int k = 0; k < kLd; ++k)
        if (load_slot(k, kLd, kMmPerSub) == n) {
          ops.ld_b(lb, k);
          ATG_PIN();
        }
    }
  }
}

template <typename Ops>
__device__ __forceinline__ void pinned_k_loop(Ops& ops, int nk) {
  using G = typename Ops::G;
  constexpr int kLd = G::kLoadsPerWave, kRdPerSub = G::kRdPerSub;
  // prologue: the panels of step 0 and, if it exists, of step 1 (which may still be in flight afterwards)
#pragma unroll
  for (int q = 0; q < kLd; ++q) ops.ld_a(0 * kLdsSlot, q);
#pragma unroll
  for (int q = 0; q < kLd; ++q) ops.ld_b(1 * kLdsSlot, q);
  // (raw barriers: __syncthreads() would add a wait for every outstanding load and store)
  if (nk > 1) {
#pragma unroll
    for (int q = 0; q < kLd; ++q) ops.ld_a(2 * kLdsSlot, q);
#pragma unroll
    for (int q = 0; q < kLd; ++q) ops.ld_b(3 * kLdsSlot, q);
    __builtin_amdgcn_s_waitcnt(0x0070 | ((2 * kLd) & 0xF) | (((2 * kLd) >> 4) << 14));   // vmcnt(2 kLd) lgkmcnt(0)
  } else {
    __builtin_amdgcn_s_waitcnt(0x0070);                                                 // vmcnt(0) lgkmcnt(0)
  }
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int n = 0; n < kRdPerSub; ++n) ops.rd(0 * kLdsSlot, 1 * kLdsSlot, 0, 0, n);
  int kt = 0, first = 0;
  for (; kt + 2 < nk; ++kt) {
    pinned_k_step<true, true>(ops, first);
    first += 2;
    if (first >= kLdsSlots) first -= kLdsSlots;
  }
  if (kt + 1 < nk) {
    pinned_k_step<true, false>(ops, first);
    first += 2;
    if (first >= kLdsSlots) first -= kLdsSlots;
  }
  pinned_k_step<false, false>(ops, first);
}

// Runs the k loop of one tile.  a_row_ptr(row) / b_row_ptr(row) return the global address of
// k = 0 of tile row `row` (0..255); rows past the operand's end must be clamped by the functor
// to some valid row (the epilogue masks them).  nk = number of 128-byte k steps (may be 0).
// Every thread of the workgroup (G::kThreads of them) must call this.  It ends with a workgroup barrier
// after the last LDS read, so the caller may reuse the LDS buffer at once.
// Fragment n of a sub-step is fetched in the order the MFMAs first need it: block row 0 of A, the block
// columns of B, then the remaining block rows of A (with two block rows, the order A0 A1 B0.. is kept).
template <typename T, typename Grid = G8, typename AF, typename BF>
__device__ __forceinline__ void gemm_tile(floatx16 (&acc)[Grid::kIB][Grid::kJB], AF a_row_ptr, BF b_row_ptr, int nk,
                                          char* smem) {
  constexpr int kIB = Grid::kIB, kJB = Grid::kJB, kLoadsPerWave = Grid::kLoadsPerWave, kRowsPerWave = Grid::kRowsPerWave;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / Grid::kWavesB, wn = wave % Grid::kWavesB;

#pragma unroll
  for (int i = 0; i < kIB; ++i)
#pragma unroll
    for (int j = 0; j < kJB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  if (nk <= 0) return;

  // direct-load sources: lane l of load q covers row wave*kRowsPerWave + q*8 + l/8, physical chunk l%8
  const char* ap[kLoadsPerWave];
  const char* bp[kLoadsPerWave];
#pragma unroll
  for (int q = 0; q < kLoadsPerWave; ++q) {
    const int row = wave * kRowsPerWave + q * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz(row);
    ap[q] = a_row_ptr(row) + c * 16;
    bp[q] = b_row_ptr(row) + c * 16;
  }
  const uint32_t wave_lds =
      __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * kRowsPerWave * kStepBytes);

  // fragment-read addresses
  int rd_a[kIB], rd_b[kJB], sw_a[kIB], sw_b[kJB];
#pragma unroll
  for (int i = 0; i < kIB; ++i) {
    const int ra = wm * (kTile / Grid::kWavesA) + i * 32 + (lane & 31);
    rd_a[i] = ra * kStepBytes;
    sw_a[i] = swz(ra) << 4;
  }
#pragma unroll
  for (int j = 0; j < kJB; ++j) {
    const int rb = wn * (kTile / Grid::kWavesB) + j * 32 + (lane & 31);
    rd_b[j] = rb * kStepBytes;
    sw_b[j] = swz(rb) << 4;
  }
  const int half16 = (lane >> 5) << 4;

  struct Ops {
    using G = Grid;
    floatx16 (&acc)[kIB][kJB];
    const char* (&ap)[kLoadsPerWave];
    const char* (&bp)[kLoadsPerWave];
    const int (&rd_a)[kIB];
    const int (&rd_b)[kJB];
    const int (&sw_a)[kIB];
    const int (&sw_b)[kJB];
    const char* smem;
    uint32_t wave_lds;
    int half16;
    uint4 fa[2][kIB], fb[2][kJB];
    __device__ __forceinline__ void mm(int f, int n) { Mma<T>::run(fa[f][n / kJB], fb[f][n % kJB], acc[n / kJB][n % kJB]); }
    __device__ __forceinline__ void rd_frag_a(int slot, int cb, int f, int i) {
      fa[f][i] = *reinterpret_cast<const uint4*>(smem + slot + rd_a[i] + (cb ^ sw_a[i]));
    }
    __device__ __forceinline__ void rd_frag_b(int slot, int cb, int f, int j) {
      fb[f][j] = *reinterpret_cast<const uint4*>(smem + slot + rd_b[j] + (cb ^ sw_b[j]));
    }
    __device__ __forceinline__ void rd(int sa, int sb, int ks, int f, int n) {
      const int cb = (ks << 5) | half16;
      if (kIB == 2) {
        if (n < kIB) rd_frag_a(sa, cb, f, n);
        else rd_frag_b(sb, cb, f, n - kIB);
      } else {
        if (n == 0) rd_frag_a(sa, cb, f, 0);
        else if (n <= kJB) rd_frag_b(sb, cb, f, n - 1);
        else rd_frag_a(sa, cb, f, n - kJB);
      }
    }
    __device__ __forceinline__ void ld_a(int slot, int q) {
      direct_load16(ap[q], wave_lds + slot + q * 8 * kStepBytes);
      ap[q] += kStepBytes;
    }
    __device__ __forceinline__ void ld_b(int slot, int q) {
      direct_load16(bp[q], wave_lds + slot + q * 8 * kStepBytes);
      bp[q] += kStepBytes;
    }
  };
  Ops ops{acc, ap, bp, rd_a, rd_b, sw_a, sw_b, smem, wave_lds, half16, {}, {}};
  pinned_k_loop(ops, nk);
}

// ------------------------------------------------------------------------------------------------
// Same tile contraction for operands stored k-major (bf16 only):
//   C[a, b] = sum_k A[k, a] * B[k, b],   A rows and B rows contiguous along a / b.
// A k-step is 64 rows of 512 bytes (256 columns) per operand.  Direct loads bring two rows per
// instruction; fragments are fetched with the transposing LDS read ds_read_b64_tr_b16: inside each
// group of 16 lanes, lane 4r + q supplies the address of 4 consecutive columns of row r (r = 0..3)
// and lane i receives column i of those four rows, i.e. 4 consecutive k for one column; two reads
// give the 8 k-values an MFMA lane needs.  The 16-byte chunk index C of row k is stored at
// (C & 16) | ((C + 4 * (k & 3)) & 15), which makes every transposing read conflict-free.
// ------------------------------------------------------------------------------------------------
typedef __bf16 bf16x4_t __attribute__((__vector_size__(4 * sizeof(__bf16))));
constexpr int kKmRows = 64;                        // k rows per step
constexpr int kKmRowBytes = kTile * 2;             // 512 bytes of columns per row

__device__ __forceinline__ uint2 lds_read_tr16(const char* p) {
  const bf16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
      (__attribute__((address_space(3))) bf16x4_t*)(__attribute__((address_space(3))) const char*)p);
  return __builtin_bit_cast(uint2, v);
}

// a0 / b0: address of element [k = 0][first column of the tile]; a_ld / b_ld: row strides in bytes;
// a_cmax / b_cmax: last 16-byte column chunk (0..31) that may be read (columns past it are fetched from
// that chunk instead and must be masked by the caller); nk: number of 64-row k-steps.
template <typename Grid = G8>
__device__ __forceinline__ void gemm_tile_kmajor(floatx16 (&acc)[Grid::kIB][Grid::kJB], const char* a0, size_t a_ld,
                                                 int a_cmax, const char* b0, size_t b_ld, int b_cmax, int nk,
                                                 char* smem) {
  constexpr int kIB = Grid::kIB, kJB = Grid::kJB, kLoadsPerWave = Grid::kLoadsPerWave;
  constexpr int kWavesA = Grid::kWavesA, kWavesB = Grid::kWavesB;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / kWavesB, wn = wave % kWavesB;

#pragma unroll
  for (int i = 0; i < kIB; ++i)
#pragma unroll
    for (int j = 0; j < kJB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  if (nk <= 0) return;

  // direct loads: instruction q of this wavefront fills rows 2*(wave*4+q), +1; lane -> (row parity, chunk)
  const char* ap[kLoadsPerWave];
  const char* bp[kLoadsPerWave];
#pragma unroll
  for (int q = 0; q < kLoadsPerWave; ++q) {
    const int k = (wave * kLoadsPerWave + q) * 2 + (lane >> 5);
    const int P = lane & 31;
    const int C = (P & 16) | ((P - 4 * (k & 3)) & 15);
    ap[q] = a0 + static_cast<size_t>(k) * a_ld + min(C, a_cmax) * 16;
    bp[q] = b0 + static_cast<size_t>(k) * b_ld + min(C, b_cmax) * 16;
  }
  const size_t a_step = a_ld * kKmRows, b_step = b_ld * kKmRows;
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * kLoadsPerWave * 1024);

  // fragment addresses: group g = lane/16 -> (column half g&1, k half g>>1); L = lane%16 -> (r, q)
  const int g = lane >> 4, L = lane & 15, r = L >> 2, qq = L & 3;
  int rd_a[kIB], rd_b[kJB];
#pragma unroll
  for (int i = 0; i < kIB; ++i) {
    const int m = wm * (kTile / kWavesA) + i * 32 + 16 * (g & 1) + 4 * qq;
    const int C = m >> 3;
    const int P = (C & 16) | ((C + 4 * r) & 15);
    rd_a[i] = (8 * (g >> 1) + r) * kKmRowBytes + P * 16 + (m & 7) * 2;
  }
#pragma unroll
  for (int j = 0; j < kJB; ++j) {
    const int m = wn * (kTile / kWavesB) + j * 32 + 16 * (g & 1) + 4 * qq;
    const int C = m >> 3;
    const int P = (C & 16) | ((C + 4 * r) & 15);
    rd_b[j] = (8 * (g >> 1) + r) * kKmRowBytes + P * 16 + (m & 7) * 2;
  }

  struct Ops {
    using G = Grid;
    floatx16 (&acc)[kIB][kJB];
    const char* (&ap)[kLoadsPerWave];
    const char* (&bp)[kLoadsPerWave];
    const int (&rd_a)[kIB];
    const int (&rd_b)[kJB];
    const char* smem;
    uint32_t wave_lds;
    size_t a_step, b_step;
    uint4 fa[2][kIB], fb[2][kJB];
    __device__ __forceinline__ void mm(int f, int n) {
      Mma<bf16_t>::run(fa[f][n / kJB], fb[f][n % kJB], acc[n / kJB][n % kJB]);
    }
    __device__ __forceinline__ void rd(int sa, int sb, int ks, int f, int n) {
      // fragment order as in gemm_tile
      bool is_a;
      int k;
      if (kIB == 2) {
        is_a = n < kIB;
        k = is_a ? n : n - kIB;
      } else {
        is_a = n == 0 || n > kJB;
        k = n == 0 ? 0 : (n <= kJB ? n - 1 : n - kJB);
      }
      const char* p = smem + ks * 16 * kKmRowBytes + (is_a ? sa + rd_a[k % kIB] : sb + rd_b[k % kJB]);
      const uint2 lo = lds_read_tr16(p);
      const uint2 hi = lds_read_tr16(p + 4 * kKmRowBytes);
      const uint4 v = make_uint4(lo.x, lo.y, hi.x, hi.y);
      if (is_a) fa[f][k % kIB] = v;
      else fb[f][k % kJB] = v;
    }
    __device__ __forceinline__ void ld_a(int slot, int q) {
      direct_load16(ap[q], wave_lds + slot + q * 1024);
      ap[q] += a_step;
    }
    __device__ __forceinline__ void ld_b(int slot, int q) {
      direct_load16(bp[q], wave_lds + slot + q * 1024);
      bp[q] += b_step;
    }
  };
  Ops ops{acc, ap, bp, rd_a, rd_b, smem, wave_lds, a_step, b_step, {}, {}};
  pinned_k_loop(ops, nk);
}

// Persistent-grid tile order.  Workgroups are dealt to the 8 XCDs round-robin by the hardware, so
// workgroup w is given the logical slot (w % 8) * (grid / 8) + w / 8: the 32 workgroups that share
// one XCD's L2 then walk neighbouring tiles.  Tiles are enumerated in bands of `band` A-tiles:
// inside a band the order runs down the band's A-tiles first, then to the next B-tile, so the
// tiles in flight form a compact patch of the output and the operand panels they stream are
// shared through L2 / Infinity Cache.
struct TileOrder {
  int n_a, n_b, band;
  __device__ __forceinline__ int total() const { return n_a * n_b; }
  __device__ __forceinline__ void decode(int t, int* ta, int* tb) const {
    const int per_band = band * n_b;
    const int bi = t / per_band;
    const int first = bi * band;
    const int rows = min(band, n_a - first);
    const int in_band = t - bi * per_band;
    *ta = first + in_band % rows;
    *tb = in_band / rows;
  }
};

__device__ __forceinline__ int logical_workgroup() {
  const int g = gridDim.x, w = blockIdx.x;
  if ((g & 7) != 0) return w;
  return (w & 7) * (g >> 3) + (w >> 3);
}

}  // namespace atg
