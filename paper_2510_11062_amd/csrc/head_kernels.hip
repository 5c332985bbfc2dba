// LM-head kernels of the AT-GRPO policy loss (gfx950).
//
// Forward (log pi_theta(y_t) inside the ratio of Eq. 2): logits tiles z[v, t] = <W[v], hidden[t]>
// are produced in MFMA accumulators, reduced to per-(vocabulary tile, token) (max, sum-exp)
// partials and the target logit, and discarded.  A small combine kernel turns the partials into
// lse and logp.
//
// Backward: logits tiles are recomputed, turned into dZ = g (onehot - softmax) in registers and
// written once, as dZ[token][vocab] in the element type of the inputs; two further contractions
// give dHidden = dZ W (k = vocab, both operands contiguous along k) and dW = dZ^T hidden
// (k = tokens, both operands read k-major through transposing LDS reads).  The fp32 path keeps a
// second, transposed copy of dZ instead.
#include <type_traits>

#include "gemm_core.hpp"
#include "head_kernels.hpp"
#include "token_kernels.hpp"

namespace atg {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ int chunk_count(const int32_t* cnt, int c0, int TC) {
  const int n = *cnt - c0;
  return n < 0 ? 0 : (n > TC ? TC : n);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ------------------------------------------------------------------------------------------------
// forward: A = W rows (vocab -> accumulator registers), B = hidden rows (tokens -> lanes)
// ------------------------------------------------------------------------------------------------
// ENT: also emit part_u, the partial sums of 2^(z log2e - m) * z that the entropy monitor needs
// (H = lse - E_p[z]); the default instantiation carries none of it.
template <typename T, bool ENT>
__global__ __launch_bounds__(kGemmThreads) void k_head_fwd(
    const T* __restrict__ hidden, const T* __restrict__ W, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cnt, int c0, const int32_t* __restrict__ token_id,
    float* __restrict__ part_m, float* __restrict__ part_s, float* __restrict__ part_u,
    float* __restrict__ zy, int H, int V, int TC, int n_vtiles, const int32_t* __restrict__ gate) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  if (gate && *gate == 0) return;
  const int n = chunk_count(cnt, c0, TC);
  if (n <= 0) return;
  const TileOrder ord{n_vtiles, (n + kTile - 1) / kTile, 8};
  const int total = ord.total();
  const TileCoord tc;
  const size_t row_bytes = static_cast<size_t>(H) * sizeof(T);
  const int nk = static_cast<int>(row_bytes / kStepBytes);
  float* red_m = reinterpret_cast<float*>(smem);          // [kWavesA][256]
  float* red_s = red_m + kWavesA * kTile;                 // [kWavesA][256]
  float* red_u = red_s + kWavesA * kTile;                 // [kWavesA][256], entropy variant only

  for (int t = logical_workgroup(); t < total; t += gridDim.x) {
    int vt, tt;
    ord.decode(t, &vt, &tt);
    const int v0 = vt * kTile, t0 = tt * kTile;

    int tcol[kJB], ycol[kJB];
#pragma unroll
    for (int j = 0; j < kJB; ++j) {
      tcol[j] = t0 + tc.b_row(j);
      ycol[j] = (tcol[j] < n) ? token_id[idx[c0 + tcol[j]]] : -1;
    }

    floatx16 acc[kIB][kJB];
    gemm_tile<T>(
        acc,
        [&](int row) {
          const int v = min(v0 + row, V - 1);
          return reinterpret_cast<const char*>(W) + static_cast<size_t>(v) * row_bytes;
        },
        [&](int row) {
          const int tk = min(t0 + row, n - 1);
          return reinterpret_cast<const char*>(hidden) + static_cast<size_t>(idx[c0 + tk]) * row_bytes;
        },
        nk, smem);

    constexpr int kWaveRows = kTile / kWavesA;   // vocab rows one wavefront holds
    const int vbase = v0 + tc.wm * kWaveRows;
    const int vrem = V - vbase;                  // rows of it that exist (may be <= 0)
    const bool ragged = vrem < kWaveRows;

#pragma unroll
    for (int j = 0; j < kJB; ++j) {
      float mx = -INFINITY;
      if (!ragged) {
#pragma unroll
        for (int i = 0; i < kIB; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[i][j][r]);
      } else {
#pragma unroll
        for (int i = 0; i < kIB; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int vl = i * 32 + 8 * (r >> 2) + 4 * tc.half + (r & 3);
            if (vl < vrem) mx = fmaxf(mx, acc[i][j][r]);
          }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m2 = (mx == -INFINITY) ? 0.f : mx * kLog2e;
      float sum = 0.f, usum = 0.f;
      if (!ragged) {
#pragma unroll
        for (int i = 0; i < kIB; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float e = fast_exp2(fmaf(acc[i][j][r], kLog2e, -m2));
            sum += e;
            if (ENT) usum = fmaf(e, acc[i][j][r], usum);
          }
      } else {
#pragma unroll
        for (int i = 0; i < kIB; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int vl = i * 32 + 8 * (r >> 2) + 4 * tc.half + (r & 3);
            if (vl < vrem) {
              const float e = fast_exp2(fmaf(acc[i][j][r], kLog2e, -m2));
              sum += e;
              if (ENT) usum = fmaf(e, acc[i][j][r], usum);
            }
          }
      }
      sum += __shfl_xor(sum, 32, 64);
      if (ENT) usum += __shfl_xor(usum, 32, 64);
      if (tc.half == 0) {
        red_m[tc.wm * kTile + tc.b_row(j)] = (mx == -INFINITY) ? -INFINITY : m2;
        red_s[tc.wm * kTile + tc.b_row(j)] = sum;
        if (ENT) red_u[tc.wm * kTile + tc.b_row(j)] = usum;
      }
      // target logit: held by exactly one lane of one wavefront of one tile
      const int rel = ycol[j] - vbase;
      const bool hit = (tcol[j] < n) && rel >= 0 && rel < kWaveRows && (((rel >> 2) & 1) == tc.half);
      if (__builtin_amdgcn_ballot_w64(hit) != 0ull) {
        float zt = 0.f;
#pragma unroll
        for (int i = 0; i < kIB; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int vl = i * 32 + 8 * (r >> 2) + (r & 3);   // half bit compared separately
            if ((rel & ~4) == vl) zt = acc[i][j][r];
          }
        if (hit) zy[tcol[j]] = zt;
      }
    }
    // fold the four vocabulary quarters of the tile: one (max, sum) per token and vocabulary tile
    barrier_lds_only();
    if (threadIdx.x < kTile && t0 + threadIdx.x < n) {
      float M = -INFINITY;
#pragma unroll
      for (int q = 0; q < kWavesA; ++q) M = fmaxf(M, red_m[q * kTile + threadIdx.x]);
      float S = 0.f, U = 0.f;
#pragma unroll
      for (int q = 0; q < kWavesA; ++q) {
        const float mq = red_m[q * kTile + threadIdx.x];
        if (mq != -INFINITY) {
          const float sc = fast_exp2(mq - M);
          S += red_s[q * kTile + threadIdx.x] * sc;
          if (ENT) U += red_u[q * kTile + threadIdx.x] * sc;
        }
      }
      part_m[static_cast<size_t>(vt) * TC + t0 + threadIdx.x] = M;
      part_s[static_cast<size_t>(vt) * TC + t0 + threadIdx.x] = S;
      if (ENT) part_u[static_cast<size_t>(vt) * TC + t0 + threadIdx.x] = U;
    }
    barrier_lds_only();   // the fold buffers are free again; the stores above need not have landed
  }
}

// ------------------------------------------------------------------------------------------------
// combine: 256 threads = 64 tokens x 4 partial slices
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_lse_combine(const int32_t* __restrict__ idx,
                                                     const int32_t* __restrict__ cnt, int c0, int TC,
                                                     int n_part, const float* __restrict__ part_m,
                                                     const float* __restrict__ part_s,
                                                     const float* __restrict__ part_u,
                                                     const float* __restrict__ zy,
                                                     float* __restrict__ logp, float* __restrict__ lse,
                                                     float* __restrict__ entropy,
                                                     const int32_t* __restrict__ gate) {
  __shared__ float sm[4][64], ss[4][64], su[4][64];
  if (gate && *gate == 0) return;
  const int n = chunk_count(cnt, c0, TC);
  const int tx = threadIdx.x & 63, py = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + tx;
  if (blockIdx.x * 64 >= n) return;
  float M = -INFINITY, S = 0.f, U = 0.f;
  if (j < n) {
    for (int p = py; p < n_part; p += 4) {
      const float m = part_m[static_cast<size_t>(p) * TC + j];
      const float s = part_s[static_cast<size_t>(p) * TC + j];
      if (m == -INFINITY) continue;
      const float Mn = fmaxf(M, m);
      const float so = fast_exp2(M - Mn), sn = fast_exp2(m - Mn);
      S = S * so + s * sn;
      if (part_u) U = U * so + part_u[static_cast<size_t>(p) * TC + j] * sn;
      M = Mn;
    }
  }
  sm[py][tx] = M;
  ss[py][tx] = S;
  su[py][tx] = U;
  __syncthreads();
  if (py == 0 && j < n) {
    float Mt = fmaxf(fmaxf(sm[0][tx], sm[1][tx]), fmaxf(sm[2][tx], sm[3][tx]));
    float St = 0.f, Ut = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (sm[q][tx] != -INFINITY) {
        const float sc = fast_exp2(sm[q][tx] - Mt);
        St += ss[q][tx] * sc;
        Ut += su[q][tx] * sc;
      }
    const float l = (Mt + __log2f(St)) * kLn2;
    const int row = idx[c0 + j];
    logp[row] = zy[j] - l;
    if (lse) lse[row] = l;
    if (entropy) entropy[row] = l - Ut / St;     // H = lse - E_p[z]
  }
}

// ------------------------------------------------------------------------------------------------
// transposes (64 x 64 tiles through LDS)
// ------------------------------------------------------------------------------------------------
// dst[c][r] = src_row(r)[c] for r < rows_valid, 0 for rows_valid <= r < rows_pad; c < cols.
// src_row(r) = src + idx[c0 + r] * src_ld when idx != null, else src + r * src_ld.
// When cnt != null, rows_valid = chunk count and rows_pad = that rounded up to 256.
template <typename T>
__global__ __launch_bounds__(256) void k_transpose(const T* __restrict__ src, int64_t src_ld,
                                                   const int32_t* __restrict__ idx,
                                                   const int32_t* __restrict__ cnt, int c0, int TC,
                                                   int rows_valid, int rows_pad, int cols,
                                                   T* __restrict__ dst, int64_t dst_ld) {
  __shared__ T tile[64][65];
  if (cnt) {
    rows_valid = chunk_count(cnt, c0, TC);
    rows_pad = (rows_valid + kTile - 1) / kTile * kTile;
  }
  const int r0 = blockIdx.x * 64, col0 = blockIdx.y * 64;
  if (r0 >= rows_pad) return;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int r = r0 + ty + 4 * k, c = col0 + tx;
    T v{};
    if (r < rows_valid && c < cols) {
      const int64_t sr = idx ? static_cast<int64_t>(idx[c0 + r]) : static_cast<int64_t>(r);
      v = src[sr * src_ld + c];
    }
    tile[ty + 4 * k][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int c = col0 + ty + 4 * k, r = r0 + tx;
    if (c < cols && r < rows_pad) dst[static_cast<int64_t>(c) * dst_ld + r] = tile[tx][ty + 4 * k];
  }
}

// ------------------------------------------------------------------------------------------------
// dZ: recompute logits, emit dZ[t][v] and dZt[v][t]
// ------------------------------------------------------------------------------------------------
template <typename T>
struct Pack4;
template <>
struct Pack4<float> {
  static __device__ __forceinline__ void store(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
  }
};
template <>
struct Pack4<bf16_t> {
  static __device__ __forceinline__ void store(bf16_t* p, float a, float b, float c, float d) {
    uint2 u;
    u.x = pack_bf16x2(a, b);
    u.y = pack_bf16x2(c, d);
    *reinterpret_cast<uint2*>(p) = u;
  }
};

constexpr int kDzRowStride = kTile * 2 + 8;              // bytes; +8 keeps the 8-byte stores conflict-free
constexpr int kDzLdsBytes = kTile * kDzRowStride;        // bf16 dZ tile staged for coalesced stores

template <typename T>
__global__ __launch_bounds__(kGemmThreads) void k_head_dz(
    const T* __restrict__ hidden, const T* __restrict__ W, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cnt, int c0, const int32_t* __restrict__ token_id,
    const float* __restrict__ lse, const float* __restrict__ coef, T* __restrict__ dZ,
    T* __restrict__ dZt, int H, int V, int Vp, int TC, int n_vtiles, const int32_t* __restrict__ gate) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  if (gate && *gate == 0) return;
  const int n = chunk_count(cnt, c0, TC);
  if (n <= 0) return;
  const TileOrder ord{n_vtiles, (n + kTile - 1) / kTile, 8};
  const int total = ord.total();
  const TileCoord tc;
  const size_t row_bytes = static_cast<size_t>(H) * sizeof(T);
  const int nk = static_cast<int>(row_bytes / kStepBytes);
  constexpr bool kStage = sizeof(T) == 2;      // bf16: dZ[t][v] goes through LDS for 16-byte stores

  for (int t = logical_workgroup(); t < total; t += gridDim.x) {
    int vt, tt;
    ord.decode(t, &vt, &tt);
    const int v0 = vt * kTile, t0 = tt * kTile;

    int tcol[kJB], ycol[kJB];
    float gcol[kJB], l2col[kJB];
#pragma unroll
    for (int j = 0; j < kJB; ++j) {
      tcol[j] = t0 + tc.b_row(j);
      if (tcol[j] < n) {
        const int row = idx[c0 + tcol[j]];
        ycol[j] = token_id[row];
        gcol[j] = coef ? coef[row] : -1.f;   // without coefficients: softmax - onehot
        l2col[j] = lse[row] * kLog2e;
      } else {
        ycol[j] = -1;
        gcol[j] = 0.f;
        l2col[j] = 0.f;
      }
    }

    floatx16 acc[kIB][kJB];
    gemm_tile<T>(
        acc,
        [&](int row) {
          const int v = min(v0 + row, V - 1);
          return reinterpret_cast<const char*>(W) + static_cast<size_t>(v) * row_bytes;
        },
        [&](int row) {
          const int tk = min(t0 + row, n - 1);
          return reinterpret_cast<const char*>(hidden) + static_cast<size_t>(idx[c0 + tk]) * row_bytes;
        },
        nk, smem);

    const int vwave = tc.wm * (kTile / kWavesA);     // first vocab row (inside the tile) of this wavefront
    // Tiles that lie fully inside the vocabulary and the token list (all but the last row / column of
    // tiles) need no per-element range checks; the target's one-hot term is rare (one element in V per
    // token) and is patched in behind a branch that is almost never taken.
    const bool interior = (v0 + kTile <= V) && (t0 + kTile <= n);
    auto emit = [&](auto guard_c) {
      constexpr bool kGuard = decltype(guard_c)::value;
#pragma unroll
      for (int j = 0; j < kJB; ++j) {
        const float g = gcol[j];
        const float nl2 = -l2col[j];
        const bool live = tcol[j] < n;
#pragma unroll
        for (int i = 0; i < kIB; ++i) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int vl = vwave + i * 32 + 8 * q + 4 * tc.half;   // first of 4 consecutive vocab rows
            const int v = v0 + vl;
            float d[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) d[e] = -g * fast_exp2(fmaf(acc[i][j][q * 4 + e], kLog2e, nl2));
            const int rel = ycol[j] - v;
            if (static_cast<unsigned>(rel) < 4u) {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (rel == e) d[e] += g;
            }
            if (kGuard) {
#pragma unroll
              for (int e = 0; e < 4; ++e) d[e] = (v + e < V && live) ? d[e] : 0.f;   // k padding, rows past the count
            }
            if (kStage) {
              uint2 u;
              u.x = pack_bf16x2(d[0], d[1]);
              u.y = pack_bf16x2(d[2], d[3]);
              *reinterpret_cast<uint2*>(smem + tc.b_row(j) * kDzRowStride + vl * 2) = u;
            } else {
              if (v < Vp) Pack4<T>::store(dZ + static_cast<size_t>(tcol[j]) * Vp + v, d[0], d[1], d[2], d[3]);
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (v + e < V) dZt[static_cast<size_t>(v + e) * TC + tcol[j]] = from_f32<T>(d[e]);
            }
          }
        }
      }
    };
    if (interior)
      emit(std::false_type{});
    else
      emit(std::true_type{});
    if (kStage) {
      __syncthreads();
      // dZ[t][v]: 32 threads x 16 bytes cover the 512 bytes of one token row of the staged tile
      const int col16 = threadIdx.x & 31;
      if (v0 + col16 * 8 < Vp) {
#pragma unroll 4
        for (int it = 0; it < kTile / 16; ++it) {
          const int row = it * 16 + (threadIdx.x >> 5);
          // two 8-byte reads per lane (rows are only 8-byte aligned); lanes 16 apart would hit the same
          // banks, so the upper half of each row takes its two halves in the opposite order
          const char* src = smem + row * kDzRowStride + col16 * 16;
          const int flip = (col16 >> 4) << 3;
          const uint2 first = *reinterpret_cast<const uint2*>(src + flip);
          const uint2 second = *reinterpret_cast<const uint2*>(src + (flip ^ 8));
          const uint2 lo = flip ? second : first;
          const uint2 hi = flip ? first : second;
          uint4 u;
          u.x = lo.x; u.y = lo.y; u.z = hi.x; u.w = hi.y;
          *reinterpret_cast<uint4*>(reinterpret_cast<char*>(dZ) +
                                    (static_cast<size_t>(t0 + row) * Vp + v0 + col16 * 8) * 2) = u;
        }
      }
      barrier_lds_only();   // every wavefront has read its part of the staged tile; its stores may still fly
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Forward and backward in one pass over the logits (bf16).  With a per-token reference c_t close
// enough to the row's largest logit, e[t][v] = exp(z[t][v] - c_t) neither overflows nor loses the
// terms that matter, and
//   lse_t = c_t + ln S_t,  S_t = sum_v e[t][v],      softmax = e / S_t,
//   dZ[t][v] = g_t (onehot - softmax) = a_t (e[t][v] - S_t [v = y_t]),  a_t = -g_t / S_t.
// The forward tile therefore writes e once (bf16, as dZ would be written), the combine step patches
// the one element per row that carries the onehot term, and the row factor a_t is applied where it is
// cheap: to the accumulators of dHidden and to the gathered hidden rows that dW contracts with.  The
// logits are not recomputed.  c_t is the target logit z[t][y_t] (one dot product per token): the
// exponent then is ln(p_v / p_y), out of range only if the sampled token is ~e^88 times less likely
// than the mode.  Rows for which S_t leaves [1, 2^60) are reported through a gate word, and the
// caller then runs the two-pass kernels for that launch instead.
// ------------------------------------------------------------------------------------------------
constexpr float kMaxRefSum = 1152921504606846976.f;   // 2^60

// c2[j] = log2(e) * <hidden[row_j], W[y_j]>: one wavefront per token of the launch
__global__ __launch_bounds__(256) void k_ref_logit(const bf16_t* __restrict__ hidden, const bf16_t* __restrict__ W,
                                                   const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt,
                                                   int c0, int TC, const int32_t* __restrict__ token_id, int H,
                                                   float* __restrict__ c2) {
  const int n = chunk_count(cnt, c0, TC);
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= n) return;
  const int row = idx[c0 + j];
  const uint4* a = reinterpret_cast<const uint4*>(hidden + static_cast<size_t>(row) * H);
  const uint4* b = reinterpret_cast<const uint4*>(W + static_cast<size_t>(token_id[row]) * H);
  float acc = 0.f;
  for (int c = lane; c < H / 8; c += 64) {
    const uint4 x = a[c], y = b[c];
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc = fmaf(__uint_as_float(xs[e] << 16), __uint_as_float(ys[e] << 16), acc);
      acc = fmaf(__uint_as_float(xs[e] & 0xffff0000u), __uint_as_float(ys[e] & 0xffff0000u), acc);
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) c2[j] = acc * kLog2e;
}

constexpr int kFeRedOffset = kDzLdsBytes;                        // staged tile, then the sums of the four vocabulary quarters
constexpr int kFeLdsBytes = kLdsBytes;
static_assert(kFeRedOffset + kWavesA * kTile * 4 <= kFeLdsBytes, "the epilogue buffers must fit the k loop's LDS");

// A = W rows (vocab -> accumulator registers), B = hidden rows (tokens -> lanes), as in the forward.
// E[j][v] = exp(z - c_j) for the tokens j of the launch; part_s[vt][j] = sum over the 256 vocabulary rows
// of tile vt; zy[j] = target logit.
__global__ __launch_bounds__(kGemmThreads) void k_head_fe(
    const bf16_t* __restrict__ hidden, const bf16_t* __restrict__ W, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cnt, int c0, const int32_t* __restrict__ token_id,
    const float* __restrict__ c2, bf16_t* __restrict__ E, float* __restrict__ part_s, float* __restrict__ zy,
    int H, int V, int Vp, int TC, int n_vtiles) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int n = chunk_count(cnt, c0, TC);
  if (n <= 0) return;
  const TileOrder ord{n_vtiles, (n + kTile - 1) / kTile, 8};
  const int total = ord.total();
  const TileCoord tc;
  const size_t row_bytes = static_cast<size_t>(H) * 2;
  const int nk = static_cast<int>(row_bytes / kStepBytes);
  float* red_s = reinterpret_cast<float*>(smem + kFeRedOffset);   // [kWavesA][256]

  for (int t = logical_workgroup(); t < total; t += gridDim.x) {
    int vt, tt;
    ord.decode(t, &vt, &tt);
    const int v0 = vt * kTile, t0 = tt * kTile;

    int tcol[kJB], ycol[kJB];
    float nc2col[kJB];
#pragma unroll
    for (int j = 0; j < kJB; ++j) {
      tcol[j] = t0 + tc.b_row(j);
      if (tcol[j] < n) {
        ycol[j] = token_id[idx[c0 + tcol[j]]];
        nc2col[j] = -c2[tcol[j]];
      } else {
        ycol[j] = -1;
        nc2col[j] = 0.f;
      }
    }

    floatx16 acc[kIB][kJB];
    gemm_tile<bf16_t>(
        acc,
        [&](int row) {
          const int v = min(v0 + row, V - 1);
          return reinterpret_cast<const char*>(W) + static_cast<size_t>(v) * row_bytes;
        },
        [&](int row) {
          const int tk = min(t0 + row, n - 1);
          return reinterpret_cast<const char*>(hidden) + static_cast<size_t>(idx[c0 + tk]) * row_bytes;
        },
        nk, smem);

    constexpr int kWaveRows = kTile / kWavesA;
    const int vwave = tc.wm * kWaveRows;             // first vocab row (inside the tile) of this wavefront
    const int vbase = v0 + vwave;

    // target logit: held by exactly one lane of one wavefront of one tile
#pragma unroll
    for (int j = 0; j < kJB; ++j) {
      const int rel = ycol[j] - vbase;
      const bool hit = (tcol[j] < n) && rel >= 0 && rel < kWaveRows && (((rel >> 2) & 1) == tc.half);
      if (__builtin_amdgcn_ballot_w64(hit) != 0ull) {
        float zt = 0.f;
#pragma unroll
        for (int i = 0; i < kIB; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int vl = i * 32 + 8 * (r >> 2) + (r & 3);   // half bit compared separately
            if ((rel & ~4) == vl) zt = acc[i][j][r];
          }
        if (hit) zy[tcol[j]] = zt;
      }
    }

    const bool interior = (v0 + kTile <= V) && (t0 + kTile <= n);
    float csum[kJB];
    auto emit = [&](auto guard_c) {
      constexpr bool kGuard = decltype(guard_c)::value;
#pragma unroll
      for (int j = 0; j < kJB; ++j) {
        const float nc2 = nc2col[j];
        const bool live = tcol[j] < n;
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < kIB; ++i) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int vl = vwave + i * 32 + 8 * q + 4 * tc.half;   // first of 4 consecutive vocab rows
            const int v = v0 + vl;
            float d[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) d[e] = fast_exp2(fmaf(acc[i][j][q * 4 + e], kLog2e, nc2));
            if (kGuard) {
#pragma unroll
              for (int e = 0; e < 4; ++e) d[e] = (v + e < V && live) ? d[e] : 0.f;   // k padding, rows past the count
            }
            sum += (d[0] + d[1]) + (d[2] + d[3]);
            uint2 u;
            u.x = pack_bf16x2(d[0], d[1]);
            u.y = pack_bf16x2(d[2], d[3]);
            *reinterpret_cast<uint2*>(smem + tc.b_row(j) * kDzRowStride + vl * 2) = u;
          }
        }
        csum[j] = sum;
      }
    };
    if (interior)
      emit(std::false_type{});
    else
      emit(std::true_type{});
#pragma unroll
    for (int j = 0; j < kJB; ++j) {
      const float sum = csum[j] + __shfl_xor(csum[j], 32, 64);
      if (tc.half == 0) red_s[tc.wm * kTile + tc.b_row(j)] = sum;
    }
    __syncthreads();
    if (threadIdx.x < kTile && t0 + threadIdx.x < n) {
      float S = 0.f;
#pragma unroll
      for (int q = 0; q < kWavesA; ++q) S += red_s[q * kTile + threadIdx.x];
      part_s[static_cast<size_t>(vt) * TC + t0 + threadIdx.x] = S;
    }
    // E[t][v]: 32 threads x 16 bytes cover the 512 bytes of one token row of the staged tile
    const int col16 = threadIdx.x & 31;
    if (v0 + col16 * 8 < Vp) {
#pragma unroll 4
      for (int it = 0; it < kTile / 16; ++it) {
        const int row = it * 16 + (threadIdx.x >> 5);
        const char* src = smem + row * kDzRowStride + col16 * 16;
        const int flip = (col16 >> 4) << 3;        // see k_head_dz: keeps the two 8-byte reads off the same banks
        const uint2 first = *reinterpret_cast<const uint2*>(src + flip);
        const uint2 second = *reinterpret_cast<const uint2*>(src + (flip ^ 8));
        const uint2 lo = flip ? second : first;
        const uint2 hi = flip ? first : second;
        uint4 u;
        u.x = lo.x; u.y = lo.y; u.z = hi.x; u.w = hi.y;
        *reinterpret_cast<uint4*>(reinterpret_cast<char*>(E) +
                                  (static_cast<size_t>(t0 + row) * Vp + v0 + col16 * 8) * 2) = u;
      }
    }
    barrier_lds_only();   // staged tile and quarter sums are free again; the stores may still fly
  }
}

// 256 threads = 64 tokens x 4 slices of the partial sums.  Per token of the launch: S, lse, logp; the
// backward coefficient g and the row factor a = -g / S; the element of E that carries the onehot term is
// replaced by e_y - S.  A row whose S is not in [.., 2^60) (overflow, NaN) or whose reference is not finite
// raises the gate and gets a = 0.
__global__ __launch_bounds__(256) void k_fe_combine(const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt,
                                                    int c0, int TC, int n_part, int head,
                                                    const float* __restrict__ part_s, const float* __restrict__ c2,
                                                    const float* __restrict__ zy,
                                                    const int32_t* __restrict__ token_id, CoefArgs ca,
                                                    float* __restrict__ logp, float* __restrict__ lse,
                                                    float* __restrict__ scale, bf16_t* __restrict__ E, int Vp,
                                                    int32_t* __restrict__ gate) {
  __shared__ float ss[4][64];
  const int n = chunk_count(cnt, c0, TC);
  const int tx = threadIdx.x & 63, py = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + tx;
  if (blockIdx.x * 64 >= n) return;
  float S = 0.f;
  if (j < n)
    for (int p = py; p < n_part; p += 4) S += part_s[static_cast<size_t>(p) * TC + j];
  ss[py][tx] = S;
  __syncthreads();
  if (py == 0 && j < n) {
    const float St = (ss[0][tx] + ss[1][tx]) + (ss[2][tx] + ss[3][tx]);
    const float c2v = c2[j];
    const float l = (c2v + __log2f(St)) * kLn2;
    const int row = idx[c0 + j];
    const float lp = zy[j] - l;
    logp[row] = lp;
    lse[row] = l;
    const bool ok = (St < kMaxRefSum) && (fabsf(c2v) < INFINITY);
    const float g = coef_value(ca, head, row, lp);
    scale[j] = ok ? -g / St : 0.f;
    const float ey = fast_exp2(fmaf(zy[j], kLog2e, -c2v));
    E[static_cast<size_t>(j) * Vp + token_id[row]] = f32_to_bf16(ey - St);
    if (!ok) atomicOr(gate, 1);
  }
}

// After the two-pass kernels have replaced a launch's E by softmax - onehot: a = -g.
__global__ __launch_bounds__(256) void k_fallback_scale(const int32_t* __restrict__ idx, const int32_t* __restrict__ cnt,
                                                        int c0, int TC, int head, CoefArgs ca,
                                                        const float* __restrict__ logp, float* __restrict__ scale,
                                                        const int32_t* __restrict__ gate) {
  if (*gate == 0) return;
  const int n = chunk_count(cnt, c0, TC);
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  const int row = idx[c0 + j];
  scale[j] = -coef_value(ca, head, row, logp[row]);
}

// Rows on the clipped branch of Eq. (2) (factor scale[j] == 0) carry no gradient.  They are taken out of the
// super-chunk before the two backward contractions: with L = number of rows with a non-zero factor, every
// such row at a position >= L (a "mover", in ascending order) is copied into the i-th position < L whose
// row has factor 0 (a "hole", in ascending order); afterwards rows 0 .. L-1 of E all carry gradient, and
// perm[j] names the row of the super-chunk that now sits at position j (its token, its factor).  Only the
// rows that fill holes move (at most min(L, n - L) of them).  One workgroup of 1024 threads, each owning a
// run of consecutive rows; sums are taken in a fixed order, so the result does not change from run to run.
constexpr int kPlanThreads = 1024;

__device__ __forceinline__ int block_exclusive_scan_1024(int v, int* lds16, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o, 64);
    if (lane >= o) incl += up;
  }
  __syncthreads();
  if (lane == 63) lds16[wave] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kPlanThreads / 64; ++w) {
    if (w < wave) base += lds16[w];
    tot += lds16[w];
  }
  *total = tot;
  return base + incl - v;
}

__global__ __launch_bounds__(kPlanThreads) void k_compact_plan(const int32_t* __restrict__ cnt, int c0, int TC,
                                                               const float* __restrict__ scale,
                                                               int32_t* __restrict__ perm, int32_t* __restrict__ holes,
                                                               int32_t* __restrict__ movers,
                                                               int32_t* __restrict__ live_cnt,
                                                               int32_t* __restrict__ pair_cnt) {
  __shared__ int lds16[kPlanThreads / 64];
  __shared__ int live_below_L;
  const int n = chunk_count(cnt, c0, TC);
  const int per = (TC + kPlanThreads - 1) / kPlanThreads;
  const int j0 = min(static_cast<int>(threadIdx.x) * per, n), j1 = min(j0 + per, n);
  int c = 0;
  for (int j = j0; j < j1; ++j) c += (scale[j] != 0.f);
  int L;
  const int before = block_exclusive_scan_1024(c, lds16, &L);   // live rows in front of this thread's run
  if (threadIdx.x == 0) live_below_L = L;                        // L == n: every row is live
  __syncthreads();
  if (j0 <= L && L < j1) {                                       // the thread that owns position L
    int lb = before;
    for (int j = j0; j < L; ++j) lb += (scale[j] != 0.f);
    live_below_L = lb;
  }
  __syncthreads();
  const int LB = live_below_L;                                   // holes = L - LB = movers
  int lb = before;
  for (int j = j0; j < j1; ++j) {
    const bool on = scale[j] != 0.f;
    if (j < L) {
      if (on) perm[j] = j;
      else holes[j - lb] = j;
    } else if (on) {
      movers[lb - LB] = j;
    }
    lb += on;
  }
  __threadfence();
  __syncthreads();
  lb = before;
  for (int j = j0; j < j1 && j < L; ++j) {
    const bool on = scale[j] != 0.f;
    if (!on) perm[j] = movers[j - lb];
    lb += on;
  }
  if (threadIdx.x == 0) {
    *live_cnt = L;
    *pair_cnt = L - LB;
  }
}

// E[holes[p]][:] = E[movers[p]][:] for p < *pair_cnt; 16 bytes per lane, one row per workgroup at a time
__global__ __launch_bounds__(256) void k_move_rows(bf16_t* __restrict__ E, int Vp, const int32_t* __restrict__ holes,
                                                   const int32_t* __restrict__ movers,
                                                   const int32_t* __restrict__ pair_cnt) {
  const int m = *pair_cnt;
  const int chunks = Vp / 8;   // 16-byte pieces per row (Vp is a multiple of 64)
  for (int p = blockIdx.x; p < m; p += gridDim.x) {
    const uint4* src = reinterpret_cast<const uint4*>(E + static_cast<size_t>(movers[p]) * Vp);
    uint4* dst = reinterpret_cast<uint4*>(E + static_cast<size_t>(holes[p]) * Vp);
    for (int c = threadIdx.x; c < chunks; c += 256) dst[c] = src[c];
  }
}

// ------------------------------------------------------------------------------------------------
// dHidden: A = dZ rows (tokens -> registers), B = Wt rows (h -> lanes), k = vocab
// ------------------------------------------------------------------------------------------------
template <typename T, typename G>
__global__ __launch_bounds__(G::kThreads) void k_head_dh(const T* __restrict__ dZ,
                                                          const T* __restrict__ Wt,
                                                          const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ cnt, int c0,
                                                          T* __restrict__ d_hidden, int H, int Vp,
                                                          int TC, const float* __restrict__ scale,
                                                          const int32_t* __restrict__ perm,
                                                          const int32_t* __restrict__ live_cnt) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // after the rows were compacted: the first *live_cnt rows of dZ, row j belonging to list position perm[j]
  const int n = perm ? min(*live_cnt, chunk_count(cnt, c0, TC)) : chunk_count(cnt, c0, TC);
  if (n <= 0) return;
  const TileOrder ord{(n + kTile - 1) / kTile, (H + kTile - 1) / kTile, 8};
  const int total = ord.total();
  const TileCoordT<G> tc;
  const size_t row_bytes = static_cast<size_t>(Vp) * sizeof(T);
  const int nk = static_cast<int>(row_bytes / kStepBytes);

  for (int t = logical_workgroup(); t < total; t += gridDim.x) {
    int tt, ht;
    ord.decode(t, &tt, &ht);
    const int t0 = tt * kTile, h0 = ht * kTile;
    floatx16 acc[G::kIB][G::kJB];
    gemm_tile<T, G>(
        acc,
        [&](int row) { return reinterpret_cast<const char*>(dZ) + static_cast<size_t>(t0 + row) * row_bytes; },
        [&](int row) {
          const int h = min(h0 + row, H - 1);
          return reinterpret_cast<const char*>(Wt) + static_cast<size_t>(h) * row_bytes;
        },
        nk, smem);
#pragma unroll
    for (int i = 0; i < G::kIB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int jt = t0 + tc.a_row(i, r);
        if (jt >= n) continue;
        const int j = perm ? perm[jt] : jt;
        T* out = d_hidden + static_cast<size_t>(idx[c0 + j]) * H;
        const float sc = scale ? scale[j] : 1.f;     // row factor of the one-pass path
#pragma unroll
        for (int jj = 0; jj < G::kJB; ++jj) {
          const int h = h0 + tc.b_row(jj);
          if (h < H) out[h] = from_f32<T>(acc[i][jj][r] * sc);
        }
      }
  }
}

// ------------------------------------------------------------------------------------------------
// dW: A = dZt rows (vocab -> registers), B = hT rows (h -> lanes), k = tokens of the super-chunk
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kGemmThreads) void k_head_dw(const T* __restrict__ dZt,
                                                          const T* __restrict__ hT,
                                                          const int32_t* __restrict__ cnt, int c0,
                                                          float* __restrict__ dW, int H, int V, int TC,
                                                          int n_vtiles, int accumulate, int first_chunk) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int n = chunk_count(cnt, c0, TC);
  if (n <= 0 && !(first_chunk && !accumulate)) return;
  const TileOrder ord{n_vtiles, (H + kTile - 1) / kTile, 8};
  const int total = ord.total();
  const TileCoord tc;
  const size_t row_bytes = static_cast<size_t>(TC) * sizeof(T);
  const int k_tokens = (n + kTile - 1) / kTile * kTile;
  const int nk = static_cast<int>(static_cast<size_t>(k_tokens) * sizeof(T) / kStepBytes);

  for (int t = logical_workgroup(); t < total; t += gridDim.x) {
    int vt, ht;
    ord.decode(t, &vt, &ht);
    const int v0 = vt * kTile, h0 = ht * kTile;
    floatx16 acc[kIB][kJB];
    gemm_tile<T>(
        acc,
        [&](int row) {
          const int v = min(v0 + row, V - 1);
          return reinterpret_cast<const char*>(dZt) + static_cast<size_t>(v) * row_bytes;
        },
        [&](int row) {
          const int h = min(h0 + row, H - 1);
          return reinterpret_cast<const char*>(hT) + static_cast<size_t>(h) * row_bytes;
        },
        nk, smem);
#pragma unroll
    for (int i = 0; i < kIB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int v = v0 + tc.a_row(i, r);
        if (v >= V) continue;
        float* out = dW + static_cast<size_t>(v) * H;
#pragma unroll
        for (int jj = 0; jj < kJB; ++jj) {
          const int h = h0 + tc.b_row(jj);
          if (h < H) out[h] = accumulate ? out[h] + acc[i][jj][r] : acc[i][jj][r];
        }
      }
  }
}

// ------------------------------------------------------------------------------------------------
// hG[j][:] = hidden[idx[c0 + j]][:] for j < n, zero rows up to the next multiple of 256 (bf16 rows
// of the super-chunk made contiguous so that the token contraction can stream them k-major)
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_gather_rows(const bf16_t* __restrict__ hidden,
                                                     const int32_t* __restrict__ idx,
                                                     const int32_t* __restrict__ cnt, int c0, int TC, int H,
                                                     const float* __restrict__ scale,
                                                     const int32_t* __restrict__ perm,
                                                     const int32_t* __restrict__ live_cnt, bf16_t* __restrict__ hG) {
  // with perm: row j of hG is list position perm[j], for j < *live_cnt
  const int n = perm ? min(*live_cnt, chunk_count(cnt, c0, TC)) : chunk_count(cnt, c0, TC);
  const int n_pad = (n + kTile - 1) / kTile * kTile;
  const int chunks = H / 8;                       // 16-byte pieces per row
  const int rows_per_block = 256 / 32;
  for (int j = blockIdx.x * rows_per_block + (threadIdx.x >> 5); j < n_pad; j += gridDim.x * rows_per_block) {
    const int jp = (j < n && perm) ? perm[j] : j;
    const uint4* src = (j < n) ? reinterpret_cast<const uint4*>(hidden + static_cast<size_t>(idx[c0 + jp]) * H) : nullptr;
    uint4* dst = reinterpret_cast<uint4*>(hG + static_cast<size_t>(j) * H);
    if (src && scale) {
      const float sc = scale[jp];
      for (int c = threadIdx.x & 31; c < chunks; c += 32) {
        const uint4 x = src[c];
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          o[e] = pack_bf16x2(__uint_as_float(xs[e] << 16) * sc, __uint_as_float(xs[e] & 0xffff0000u) * sc);
        dst[c] = make_uint4(o[0], o[1], o[2], o[3]);
      }
    } else {
      for (int c = threadIdx.x & 31; c < chunks; c += 32) dst[c] = src ? src[c] : make_uint4(0, 0, 0, 0);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// dW (bf16): dW[v][h] (+)= sum_t dZ[t][v] * hG[t][h], both operands read k-major (no transposed
// copies): A = dZ columns (vocab -> registers), B = hG columns (h -> lanes), k = tokens
// ------------------------------------------------------------------------------------------------
template <typename G>
__global__ __launch_bounds__(G::kThreads) void k_head_dw_km(const bf16_t* __restrict__ dZ,
                                                             const bf16_t* __restrict__ hG,
                                                             const int32_t* __restrict__ cnt, int c0,
                                                             float* __restrict__ dW, int H, int V, int Vp,
                                                             int TC, int n_vtiles, int accumulate,
                                                             int first_chunk, const int32_t* __restrict__ live_cnt) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // live_cnt: the rows were compacted, only the first *live_cnt of the chunk take part
  const int n = live_cnt ? min(*live_cnt, chunk_count(cnt, c0, TC)) : chunk_count(cnt, c0, TC);
  if (n <= 0 && !(first_chunk && !accumulate)) return;
  // bands of 32 / (tiles along H) vocabulary tiles: the 32 workgroups that share an XCD's L2 then cover every
  // H-tile of the same few vocabulary tiles, and each panel of the large operand (the 10 GB of dZ rows)
  // is fetched by one XCD only (measured 2.4 % faster than bands of 8)
  const int n_htiles = (H + kTile - 1) / kTile;
  const TileOrder ord{n_vtiles, n_htiles, max(1, 32 / n_htiles)};
  const int total = ord.total();
  const TileCoordT<G> tc;
  const int nk = (n + kTile - 1) / kTile * kTile / kKmRows;

  for (int t = logical_workgroup(); t < total; t += gridDim.x) {
    int vt, ht;
    ord.decode(t, &vt, &ht);
    const int v0 = vt * kTile, h0 = ht * kTile;
    floatx16 acc[G::kIB][G::kJB];
    gemm_tile_kmajor<G>(acc, reinterpret_cast<const char*>(dZ + v0), static_cast<size_t>(Vp) * 2,
                     min(31, (Vp - v0) / 8 - 1), reinterpret_cast<const char*>(hG + h0),
                     static_cast<size_t>(H) * 2, min(31, (H - h0) / 8 - 1), nk, smem);
#pragma unroll
    for (int i = 0; i < G::kIB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int v = v0 + tc.a_row(i, r);
        if (v >= V) continue;
        float* out = dW + static_cast<size_t>(v) * H;
#pragma unroll
        for (int jj = 0; jj < G::kJB; ++jj) {
          const int h = h0 + tc.b_row(jj);
          if (h < H) out[h] = accumulate ? out[h] + acc[i][jj][r] : acc[i][jj][r];
        }
      }
  }
}

template <typename K>
int allow_big_lds(K kernel, int bytes = kLdsBytes) {
  ATG_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  return AT_GRPO_OK;
}

int gemm_grid() {
  int cus = device_cu_count();
  if (cus <= 0) cus = 256;
  return cus;
}

}  // namespace

// ================================================================================================
// launchers
// ================================================================================================
template <typename T, bool ENT>
int launch_head_fwd_t(const HeadGeom& g, const HeadChunk& ch, const void* hidden, const void* W,
                      const int32_t* token_id, float* part_m, float* part_s, float* part_u, float* zy,
                      hipStream_t s, const int32_t* gate) {
  auto k = k_head_fwd<T, ENT>;
  ATG_TRY(allow_big_lds(k));
  hipLaunchKernelGGL(k, dim3(gemm_grid()), dim3(kGemmThreads), kLdsBytes, s, static_cast<const T*>(hidden),
                     static_cast<const T*>(W), ch.idx, ch.cnt, ch.c0, token_id, part_m, part_s, part_u, zy, g.H,
                     g.V, g.TC, g.n_vtiles, gate);
  return AT_GRPO_OK;
}

int launch_head_fwd(const HeadGeom& g, const HeadChunk& ch, const void* hidden, const void* W,
                    const int32_t* token_id, float* part_m, float* part_s, float* part_u, float* zy,
                    hipStream_t s, const int32_t* gate) {
  ProfScope ps(PROF_HEAD_FWD, s);
  if (g.dtype == AT_GRPO_BF16) {
    if (part_u) ATG_TRY((launch_head_fwd_t<bf16_t, true>(g, ch, hidden, W, token_id, part_m, part_s, part_u, zy, s, gate)));
    else ATG_TRY((launch_head_fwd_t<bf16_t, false>(g, ch, hidden, W, token_id, part_m, part_s, part_u, zy, s, gate)));
  } else {
    if (part_u) ATG_TRY((launch_head_fwd_t<float, true>(g, ch, hidden, W, token_id, part_m, part_s, part_u, zy, s, gate)));
    else ATG_TRY((launch_head_fwd_t<float, false>(g, ch, hidden, W, token_id, part_m, part_s, part_u, zy, s, gate)));
  }
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_lse_combine(const HeadGeom& g, const HeadChunk& ch, const float* part_m, const float* part_s,
                       const float* part_u, const float* zy, float* logp, float* lse, float* entropy,
                       hipStream_t s, const int32_t* gate) {
  ProfScope ps(PROF_LSE_COMBINE, s);
  hipLaunchKernelGGL(k_lse_combine, dim3(g.TC / 64), dim3(256), 0, s, ch.idx, ch.cnt, ch.c0, g.TC,
                     g.n_vtiles, part_m, part_s, part_u, zy, logp, lse, part_u ? entropy : nullptr, gate);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_transpose_w(const HeadGeom& g, const void* W, void* Wt, hipStream_t s) {
  ProfScope ps(PROF_TRANSPOSE, s);
  dim3 grid(static_cast<unsigned>(ceil_div(g.Vp, 64)), static_cast<unsigned>(ceil_div(g.H, 64)));
  if (g.dtype == AT_GRPO_BF16)
    hipLaunchKernelGGL(k_transpose<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t*>(W),
                       static_cast<int64_t>(g.H), nullptr, nullptr, 0, 0, g.V, g.Vp, g.H,
                       static_cast<bf16_t*>(Wt), static_cast<int64_t>(g.Vp));
  else
    hipLaunchKernelGGL(k_transpose<float>, grid, dim3(256), 0, s, static_cast<const float*>(W),
                       static_cast<int64_t>(g.H), nullptr, nullptr, 0, 0, g.V, g.Vp, g.H,
                       static_cast<float*>(Wt), static_cast<int64_t>(g.Vp));
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_gather_transpose_hidden(const HeadGeom& g, const HeadChunk& ch, const void* hidden, void* hT,
                                   hipStream_t s, const float* scale, const int32_t* perm, const int32_t* live_cnt) {
  ProfScope ps(PROF_TRANSPOSE, s);
  if (g.dtype == AT_GRPO_BF16) {
    // bf16: plain row gather (the token contraction reads it k-major)
    hipLaunchKernelGGL(k_gather_rows, dim3(2048), dim3(256), 0, s, static_cast<const bf16_t*>(hidden), ch.idx,
                       ch.cnt, ch.c0, g.TC, g.H, scale, perm, live_cnt, static_cast<bf16_t*>(hT));
  } else {
    dim3 grid(static_cast<unsigned>(g.TC / 64), static_cast<unsigned>(ceil_div(g.H, 64)));
    hipLaunchKernelGGL(k_transpose<float>, grid, dim3(256), 0, s, static_cast<const float*>(hidden),
                       static_cast<int64_t>(g.H), ch.idx, ch.cnt, ch.c0, g.TC, 0, 0, g.H,
                       static_cast<float*>(hT), static_cast<int64_t>(g.TC));
  }
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_head_dz(const HeadGeom& g, const HeadChunk& ch, const void* hidden, const void* W,
                   const int32_t* token_id, const float* lse, const float* coef, void* dZ, void* dZt,
                   hipStream_t s, const int32_t* gate) {
  ProfScope ps(PROF_HEAD_DZ, s);
  if (g.dtype == AT_GRPO_BF16) {
    auto k = k_head_dz<bf16_t>;
    constexpr int lds = kDzLdsBytes > kLdsBytes ? kDzLdsBytes : kLdsBytes;
    ATG_TRY(allow_big_lds(k, lds));
    hipLaunchKernelGGL(k, dim3(gemm_grid()), dim3(kGemmThreads), lds, s,
                       static_cast<const bf16_t*>(hidden), static_cast<const bf16_t*>(W), ch.idx, ch.cnt,
                       ch.c0, token_id, lse, coef, static_cast<bf16_t*>(dZ), static_cast<bf16_t*>(dZt),
                       g.H, g.V, g.Vp, g.TC, g.n_vtiles, gate);
  } else {
    auto k = k_head_dz<float>;
    ATG_TRY(allow_big_lds(k));
    hipLaunchKernelGGL(k, dim3(gemm_grid()), dim3(kGemmThreads), kLdsBytes, s,
                       static_cast<const float*>(hidden), static_cast<const float*>(W), ch.idx, ch.cnt,
                       ch.c0, token_id, lse, coef, static_cast<float*>(dZ), static_cast<float*>(dZt), g.H,
                       g.V, g.Vp, g.TC, g.n_vtiles, gate);
  }
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_ref_logit(const HeadGeom& g, const HeadChunk& ch, const void* hidden, const void* W,
                     const int32_t* token_id, float* c2, hipStream_t s) {
  ProfScope ps(PROF_LSE_COMBINE, s);
  if (g.dtype != AT_GRPO_BF16) return AT_GRPO_EUNSUPPORTED;
  hipLaunchKernelGGL(k_ref_logit, dim3(g.TC / 4), dim3(256), 0, s, static_cast<const bf16_t*>(hidden),
                     static_cast<const bf16_t*>(W), ch.idx, ch.cnt, ch.c0, g.TC, token_id, g.H, c2);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_head_fe(const HeadGeom& g, const HeadChunk& ch, const void* hidden, const void* W,
                   const int32_t* token_id, const float* c2, void* E, float* part_s, float* zy, hipStream_t s) {
  ProfScope ps(PROF_HEAD_FE, s);
  if (g.dtype != AT_GRPO_BF16) return AT_GRPO_EUNSUPPORTED;
  auto k = k_head_fe;
  ATG_TRY(allow_big_lds(k, kFeLdsBytes));
  hipLaunchKernelGGL(k, dim3(gemm_grid()), dim3(kGemmThreads), kFeLdsBytes, s, static_cast<const bf16_t*>(hidden),
                     static_cast<const bf16_t*>(W), ch.idx, ch.cnt, ch.c0, token_id, c2, static_cast<bf16_t*>(E),
                     part_s, zy, g.H, g.V, g.Vp, g.TC, g.n_vtiles);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_fe_combine(const HeadGeom& g, const HeadChunk& ch, int head, const float* part_s, const float* c2,
                      const float* zy, const int32_t* token_id, const CoefArgs& ca, float* logp, float* lse,
                      float* scale, void* E, int32_t* gate, hipStream_t s) {
  ProfScope ps(PROF_LSE_COMBINE, s);
  hipLaunchKernelGGL(k_fe_combine, dim3(g.TC / 64), dim3(256), 0, s, ch.idx, ch.cnt, ch.c0, g.TC, g.n_vtiles,
                     head, part_s, c2, zy, token_id, ca, logp, lse, scale, static_cast<bf16_t*>(E), g.Vp, gate);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_fallback_scale(const HeadGeom& g, const HeadChunk& ch, int head, const CoefArgs& ca, const float* logp,
                          float* scale, const int32_t* gate, hipStream_t s) {
  ProfScope ps(PROF_COEF, s);
  hipLaunchKernelGGL(k_fallback_scale, dim3(g.TC / 256), dim3(256), 0, s, ch.idx, ch.cnt, ch.c0, g.TC, head, ca,
                     logp, scale, gate);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_compact_rows(const HeadGeom& g, const HeadChunk& ch, const float* scale, void* E, int32_t* perm,
                        int32_t* holes, int32_t* movers, int32_t* live_cnt, int32_t* pair_cnt, hipStream_t s) {
  ProfScope ps(PROF_COEF, s);
  if (g.dtype != AT_GRPO_BF16 || g.TC > 32 * kPlanThreads) return AT_GRPO_EUNSUPPORTED;
  hipLaunchKernelGGL(k_compact_plan, dim3(1), dim3(kPlanThreads), 0, s, ch.cnt, ch.c0, g.TC, scale, perm, holes,
                     movers, live_cnt, pair_cnt);
  ATG_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_move_rows, dim3(2048), dim3(256), 0, s, static_cast<bf16_t*>(E), g.Vp, holes, movers, pair_cnt);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_head_dh(const HeadGeom& g, const HeadChunk& ch, const void* dZ, const void* Wt, void* d_hidden,
                   hipStream_t s, const float* scale, const int32_t* perm, const int32_t* live_cnt) {
  ProfScope ps(PROF_HEAD_DH, s);
  if (g.dtype == AT_GRPO_BF16) {
    auto k = k_head_dh<bf16_t, G4>;   // k = vocabulary: long loop, 4 wavefronts of 128 x 128
    ATG_TRY(allow_big_lds(k));
    hipLaunchKernelGGL(k, dim3(gemm_grid()), dim3(G4::kThreads), kLdsBytes, s,
                       static_cast<const bf16_t*>(dZ), static_cast<const bf16_t*>(Wt), ch.idx, ch.cnt, ch.c0,
                       static_cast<bf16_t*>(d_hidden), g.H, g.Vp, g.TC, scale, perm, live_cnt);
  } else {
    auto k = k_head_dh<float, G8>;
    ATG_TRY(allow_big_lds(k));
    hipLaunchKernelGGL(k, dim3(gemm_grid()), dim3(kGemmThreads), kLdsBytes, s,
                       static_cast<const float*>(dZ), static_cast<const float*>(Wt), ch.idx, ch.cnt, ch.c0,
                       static_cast<float*>(d_hidden), g.H, g.Vp, g.TC, scale, perm, live_cnt);
  }
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_head_dw(const HeadGeom& g, const HeadChunk& ch, const void* dZ, const void* dZt, const void* hT,
                   float* dW, int accumulate, int first_chunk, hipStream_t s, const int32_t* live_cnt) {
  ProfScope ps(PROF_HEAD_DW, s);
  if (g.dtype == AT_GRPO_BF16) {
    auto k = k_head_dw_km<G8>;        // 8 wavefronts: measured 4 % faster here than the 4-wavefront layout
    ATG_TRY(allow_big_lds(k));
    hipLaunchKernelGGL(k, dim3(gemm_grid()), dim3(G8::kThreads), kLdsBytes, s, static_cast<const bf16_t*>(dZ),
                       static_cast<const bf16_t*>(hT), ch.cnt, ch.c0, dW, g.H, g.V, g.Vp, g.TC, g.n_vtiles,
                       accumulate, first_chunk, live_cnt);
  } else {
    auto k = k_head_dw<float>;
    ATG_TRY(allow_big_lds(k));
    hipLaunchKernelGGL(k, dim3(gemm_grid()), dim3(kGemmThreads), kLdsBytes, s,
                       static_cast<const float*>(dZt), static_cast<const float*>(hT), ch.cnt, ch.c0, dW, g.H,
                       g.V, g.TC, g.n_vtiles, accumulate, first_chunk);
  }
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

}  // namespace atg
