// Shared host/device helpers of the AT-GRPO policy-loss library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "at_grpo.h"

namespace atg {

#define ATG_HIP_TRY(expr)                         \
  do {                                            \
    hipError_t atg_e_ = (expr);                   \
    if (atg_e_ != hipSuccess) return AT_GRPO_EHIP; \
  } while (0)

#define ATG_LAUNCH_CHECK() ATG_HIP_TRY(hipGetLastError())

#define ATG_TRY(expr)                  \
  do {                                 \
    int atg_s_ = (expr);               \
    if (atg_s_ != AT_GRPO_OK) return atg_s_; \
  } while (0)

constexpr int kMaxHeads = 16;
constexpr int kWave = 64;

// Storage type of a bf16 element (bit pattern only; arithmetic happens in fp32).
struct bf16_t {
  uint16_t bits;
};

inline size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Bump allocator over the caller's workspace.  With base == nullptr it only measures.
struct WsAlloc {
  char* base;
  size_t off;
  explicit WsAlloc(void* b) : base(static_cast<char*>(b)), off(0) {}
  template <typename T>
  T* take(size_t count) {
    off = round_up(off, 256);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
  size_t bytes() const { return round_up(off, 256); }
};

// ---- optional per-kernel timing (see at_grpo_profile_* in the header) -------------------------
enum ProfClass {
  PROF_GROUP = 0,      // grouping + advantage kernels
  PROF_PREP,           // token routing, flags, compaction
  PROF_HEAD_FWD,       // head contraction + online softmax partials
  PROF_LSE_COMBINE,    // partial (max, sum) -> lse, logp
  PROF_SURROGATE,      // ratio, clip, masked reduction
  PROF_COEF,           // backward coefficient g_t
  PROF_TRANSPOSE,      // W^T and gathered hidden^T
  PROF_HEAD_DZ,        // logits recompute + dZ
  PROF_HEAD_DH,        // dHidden = dZ W
  PROF_HEAD_DW,        // dW = dZ^T hidden
  PROF_FILL,           // buffer clears
  PROF_GRAD_NORM,      // global gradient norm of the head update
  PROF_ADAM,           // fused clip + Adam step
  PROF_HEAD_FE,        // head contraction that writes the exponentials (one-pass forward + backward)
  PROF_N
};

void prof_begin(int cls, hipStream_t s);
void prof_end(int cls, hipStream_t s);

struct ProfScope {
  int cls;
  hipStream_t s;
  ProfScope(int c, hipStream_t st) : cls(c), s(st) { prof_begin(cls, s); }
  ~ProfScope() { prof_end(cls, s); }
};

int device_cu_count();

#ifdef __HIPCC__
// ---- device helpers ------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(static_cast<uint32_t>(v.bits) << 16); }

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  // round to nearest even; NaN stays NaN
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return bf16_t{static_cast<uint16_t>((u >> 16) | 0x40)};
  u += 0x7fffu + ((u >> 16) & 1u);
  return bf16_t{static_cast<uint16_t>(u >> 16)};
}

// two floats -> packed bf16 pair (low half = a), round to nearest even in hardware (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

template <typename T>
__device__ __forceinline__ T from_f32(float f);
template <>
__device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) { return f32_to_bf16(f); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;   // valid in lane 0
}

__device__ __forceinline__ int wave_sum_int(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

// Sum over a 256-thread block in a fixed order; result valid in every thread.
__device__ __forceinline__ float block_sum_256(float v, float* lds4) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) lds4[wave] = v;
  __syncthreads();
  return (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
}

__device__ __forceinline__ int block_sum_256_int(int v, int* lds4) {
  v = wave_sum_int(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) lds4[wave] = v;
  __syncthreads();
  return lds4[0] + lds4[1] + lds4[2] + lds4[3];
}

// Exclusive scan of one int per thread over a 256-thread block; *total gets the block sum.
__device__ __forceinline__ int block_exclusive_scan_256(int v, int* lds4, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int up = __shfl_up(incl, o, 64);
    if (lane >= o) incl += up;
  }
  __syncthreads();
  if (lane == 63) lds4[wave] = incl;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (w < wave) base += lds4[w];
  *total = lds4[0] + lds4[1] + lds4[2] + lds4[3];
  return base + incl - v;
}
#endif  // __HIPCC__

}  // namespace atg
