// Workgroup-tile contraction on the gfx950 matrix cores.
//
// One 256-thread workgroup (4 wavefronts, 2 x 2) produces a 256 x 256 fp32 tile
//   C[a, b] = sum_k A[a, k] * B[b, k]
// from two operands that are both contiguous along k ("NT" layout).  Each wavefront owns a
// 128 x 128 sub-tile held as 4 x 4 MFMA 32x32 accumulator blocks (256 accumulator registers per
// lane).  k is consumed in steps of 128 bytes per row (64 bf16 or 32 fp32 elements): the step's
// 256 + 256 row segments are staged through LDS, double buffered, with an XOR swizzle of the
// 16-byte chunk index so that both the staging stores and the ds_read_b128 fragment loads are
// free of bank conflicts.
//
// Accumulator layout (per lane, block (i, j), register r = 0..15):
//   a = wm*128 + i*32 + 8*(r/4) + 4*(lane/32) + (r%4)        (A row inside the tile)
//   b = wn*128 + j*32 + lane%32                               (B row inside the tile)
#pragma once

#include "common.hpp"

namespace atg {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int kTile = 256;                       // rows of each operand per tile
constexpr int kStepBytes = 128;                  // bytes of k per row per step
constexpr int kGemmThreads = 256;
constexpr int kLdsOperand = kTile * kStepBytes;  // 32 KiB
constexpr int kLdsStage = 2 * kLdsOperand;       // A then B
constexpr int kLdsBytes = 2 * kLdsStage;         // two stages: 128 KiB

__device__ __forceinline__ int swz16(int row) { return ((row ^ (row >> 3)) & 7) << 4; }

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

struct TileCoord {
  int lane, wm, wn, half;
  __device__ __forceinline__ TileCoord() {
    lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    wm = wave >> 1;
    wn = wave & 1;
    half = lane >> 5;
  }
  // A row (inside the tile) of accumulator register r of block row i
  __device__ __forceinline__ int a_row(int i, int r) const {
    return wm * 128 + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
  }
  // B row (inside the tile) of block column j
  __device__ __forceinline__ int b_row(int j) const { return wn * 128 + j * 32 + (lane & 31); }
};

// Runs the k loop of one tile.  a_row_ptr(row) / b_row_ptr(row) return the global address of
// k = 0 of tile row `row` (0..255); rows past the operand's end must be clamped by the functor
// to some valid row (the epilogue masks them).  nk = number of 128-byte k steps (may be 0).
// Every thread of the workgroup must call this; it ends with a workgroup barrier.
template <typename T, typename AF, typename BF>
__device__ __forceinline__ void gemm_tile(floatx16 (&acc)[4][4], AF a_row_ptr, BF b_row_ptr, int nk,
                                          char* smem) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int ld_row = tid >> 3, ld_chunk = tid & 7;

  const char* ap[8];
  const char* bp[8];
  int st_off[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = ld_row + 32 * i;
    ap[i] = a_row_ptr(row) + ld_chunk * 16;
    bp[i] = b_row_ptr(row) + ld_chunk * 16;
    st_off[i] = row * kStepBytes + ((ld_chunk << 4) ^ swz16(row));
  }
  int rd_a[4], rd_b[4], sw_a[4], sw_b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ra = wm * 128 + i * 32 + (lane & 31);
    const int rb = wn * 128 + i * 32 + (lane & 31);
    rd_a[i] = ra * kStepBytes;
    rd_b[i] = kLdsOperand + rb * kStepBytes;
    sw_a[i] = swz16(ra);
    sw_b[i] = swz16(rb);
  }

#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  if (nk <= 0) {
    __syncthreads();
    return;
  }

  uint4 ga[8], gb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    ga[i] = *reinterpret_cast<const uint4*>(ap[i]);
    gb[i] = *reinterpret_cast<const uint4*>(bp[i]);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    *reinterpret_cast<uint4*>(smem + st_off[i]) = ga[i];
    *reinterpret_cast<uint4*>(smem + kLdsOperand + st_off[i]) = gb[i];
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * kLdsStage;
    char* nxt = smem + ((kt + 1) & 1) * kLdsStage;
    const bool more = (kt + 1 < nk);
    if (more) {
      const size_t kb = static_cast<size_t>(kt + 1) * kStepBytes;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        ga[i] = *reinterpret_cast<const uint4*>(ap[i] + kb);
        gb[i] = *reinterpret_cast<const uint4*>(bp[i] + kb);
      }
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int cb = (ks * 2 + (lane >> 5)) << 4;
      uint4 fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        fa[i] = *reinterpret_cast<const uint4*>(cur + rd_a[i] + (cb ^ sw_a[i]));
        fb[i] = *reinterpret_cast<const uint4*>(cur + rd_b[i] + (cb ^ sw_b[i]));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) Mma<T>::run(fa[i], fb[j], acc[i][j]);
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        *reinterpret_cast<uint4*>(nxt + st_off[i]) = ga[i];
        *reinterpret_cast<uint4*>(nxt + kLdsOperand + st_off[i]) = gb[i];
      }
    }
    __syncthreads();
  }
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
