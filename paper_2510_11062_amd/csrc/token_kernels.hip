// Per-token streaming kernels of the AT-GRPO policy loss (gfx950): routing rows to responses and
// heads (the per-model batches B_m of Sec. 3), stable compaction, the clipped surrogate of
// Eq. (2) with a fixed-order reduction, and the backward coefficient d loss / d logp.
#include "token_kernels.hpp"

namespace atg {

namespace {

__global__ void k_fill_i32(int32_t* __restrict__ p, int64_t n, int32_t value) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride)
    p[i] = value;
}

__global__ void k_zero16(uint4* __restrict__ p, int64_t n16) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  const uint4 z = make_uint4(0, 0, 0, 0);
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride)
    p[i] = z;
}

__device__ __forceinline__ int head_of_response(int r, int n_heads, int n_agent,
                                                const int32_t* resp_agent,
                                                const int32_t* head_of_agent, int32_t* err) {
  if (n_heads == 1 || resp_agent == nullptr || head_of_agent == nullptr) return 0;
  const int a = resp_agent[r];
  if (a < 0 || a >= n_agent) {
    atomicOr(err, AT_GRPO_DATA_AGENT_RANGE);
    return -1;
  }
  const int h = head_of_agent[a];
  if (h < 0 || h >= n_heads) {
    atomicOr(err, AT_GRPO_DATA_AGENT_RANGE);
    return -1;
  }
  return h;
}

// one wavefront per response
__global__ __launch_bounds__(256) void k_route(TokenLayout L, int32_t* __restrict__ err,
                                               int32_t* __restrict__ resp_of_tok,
                                               int32_t* __restrict__ flag) {
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int n_waves = (gridDim.x * blockDim.x) >> 6;
  for (int r = wave; r < L.n_resp; r += n_waves) {
    const int64_t lo = L.cu_seqlens[r], hi = L.cu_seqlens[r + 1];
    if (lo < 0 || hi < lo || hi > L.n_tok) {
      if (lane == 0) atomicOr(err, AT_GRPO_DATA_SEQLENS);
      continue;
    }
    const int head = head_of_response(r, L.n_heads, L.n_agent, L.resp_agent, L.head_of_agent, err);
    for (int64_t t = lo + lane; t < hi; t += 64) {
      bool on = (head >= 0) && (L.mask == nullptr || L.mask[t] != 0);
      if (on && L.token_id != nullptr) {
        const int y = L.token_id[t];
        if (y < 0 || y >= L.V) {
          atomicOr(err, AT_GRPO_DATA_TOKEN_RANGE);
          on = false;
        }
      }
      resp_of_tok[t] = r;
      flag[t] = on ? head : -1;
    }
  }
}

__global__ __launch_bounds__(256) void k_count(const int32_t* __restrict__ flag, int64_t n_tok,
                                               int n_heads, int64_t n_blk,
                                               int32_t* __restrict__ blk_cnt) {
  __shared__ int lds4[4];
  const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kTokPerBlock + threadIdx.x * 8;
  int f[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = (t0 + e < n_tok) ? flag[t0 + e] : -1;
  for (int m = 0; m < n_heads; ++m) {
    int c = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) c += (f[e] == m);
    const int tot = block_sum_256_int(c, lds4);
    if (threadIdx.x == 0) blk_cnt[m * n_blk + blockIdx.x] = tot;
  }
}

// single block: exclusive scan of the per-block counts of every head
__global__ __launch_bounds__(256) void k_scan_blocks(const int32_t* __restrict__ blk_cnt, int n_heads,
                                                     int64_t n_blk, int32_t* __restrict__ blk_off,
                                                     int32_t* __restrict__ cnt) {
  __shared__ int lds4[4];
  for (int m = 0; m < n_heads; ++m) {
    int running = 0;
    for (int64_t base = 0; base < n_blk; base += 256) {
      const int64_t b = base + threadIdx.x;
      const int v = (b < n_blk) ? blk_cnt[m * n_blk + b] : 0;
      int tot;
      const int ex = block_exclusive_scan_256(v, lds4, &tot);
      if (b < n_blk) blk_off[m * n_blk + b] = running + ex;
      running += tot;
    }
    if (threadIdx.x == 0) cnt[m] = running;
  }
  for (int m = n_heads + threadIdx.x; m < kMaxHeads; m += 256) cnt[m] = 0;
}

__global__ __launch_bounds__(256) void k_scatter(const int32_t* __restrict__ flag, int64_t n_tok,
                                                 int n_heads, int64_t n_blk,
                                                 const int32_t* __restrict__ blk_off,
                                                 int32_t* __restrict__ idx) {
  __shared__ int lds4[4];
  const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kTokPerBlock + threadIdx.x * 8;
  int f[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = (t0 + e < n_tok) ? flag[t0 + e] : -1;
  for (int m = 0; m < n_heads; ++m) {
    int c = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) c += (f[e] == m);
    int tot;
    int pos = blk_off[m * n_blk + blockIdx.x] + block_exclusive_scan_256(c, lds4, &tot);
    int32_t* out = idx + static_cast<int64_t>(m) * n_tok;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (f[e] == m) out[pos++] = static_cast<int32_t>(t0 + e);
  }
}

// one wavefront per response: participating rows of the response
__global__ __launch_bounds__(256) void k_resp_len(TokenLayout L, const int32_t* __restrict__ flag,
                                                  int32_t* __restrict__ resp_len) {
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int n_waves = (gridDim.x * blockDim.x) >> 6;
  for (int r = wave; r < L.n_resp; r += n_waves) {
    const int64_t lo = L.cu_seqlens[r], hi = L.cu_seqlens[r + 1];
    int c = 0;
    if (!(lo < 0 || hi < lo || hi > L.n_tok))
      for (int64_t t = lo + lane; t < hi; t += 64) c += (flag[t] >= 0);
    c = wave_sum_int(c);
    if (lane == 0) resp_len[r] = c;
  }
}

// single block: responses with at least one participating row, per head
__global__ __launch_bounds__(256) void k_resp_cnt(TokenLayout L, const int32_t* __restrict__ resp_len,
                                                  int32_t* __restrict__ err,
                                                  int32_t* __restrict__ resp_cnt) {
  __shared__ int lds4[4];
  for (int m = 0; m < L.n_heads; ++m) {
    int c = 0;
    for (int r = threadIdx.x; r < L.n_resp; r += 256)
      if (resp_len[r] > 0 &&
          head_of_response(r, L.n_heads, L.n_agent, L.resp_agent, L.head_of_agent, err) == m)
        ++c;
    const int tot = block_sum_256_int(c, lds4);
    if (threadIdx.x == 0) resp_cnt[m] = tot;
  }
}

// LPR lanes per response (64, 32 or 16, chosen from the mean response length): every row of the
// response is read once (logp, old_logp, mask, and token_id when given) in 4-row vectors, its clip
// flags are written, and the response's sum of surrogate terms and its count of participating rows
// are reduced in a fixed order.  Needs no per-row routing arrays: the advantage and the head are
// per-response scalars.
template <int LPR>
__global__ __launch_bounds__(256) void k_surrogate_resp(TokenLayout L, const float* __restrict__ logp,
                                                        const float* __restrict__ old_logp,
                                                        const float* __restrict__ adv, ClipConst cc, int agg,
                                                        uint8_t* __restrict__ clip_mask,
                                                        float* __restrict__ resp_sum,
                                                        int32_t* __restrict__ resp_cnt,
                                                        int32_t* __restrict__ resp_head,
                                                        int32_t* __restrict__ err) {
  const int lane = threadIdx.x & (LPR - 1);
  const int team = (blockIdx.x * blockDim.x + threadIdx.x) / LPR;
  const int n_teams = (gridDim.x * blockDim.x) / LPR;
  for (int r = team; r < L.n_resp; r += n_teams) {
    const int64_t lo = L.cu_seqlens[r], hi = L.cu_seqlens[r + 1];
    if (lo < 0 || hi < lo || hi > L.n_tok) {
      if (lane == 0) {
        atomicOr(err, AT_GRPO_DATA_SEQLENS);
        resp_sum[r] = 0.f;
        resp_cnt[r] = 0;
        resp_head[r] = -1;
      }
      continue;
    }
    const int head = head_of_response(r, L.n_heads, L.n_agent, L.resp_agent, L.head_of_agent, err);
    const float A = adv[r];
    float sum = 0.f;
    int cnt = 0;
    auto one = [&](int64_t t) {
      bool on = (head >= 0) && (L.mask == nullptr || L.mask[t] != 0);
      if (on && L.token_id != nullptr) {
        const int y = L.token_id[t];
        if (y < 0 || y >= L.V) {
          atomicOr(err, AT_GRPO_DATA_TOKEN_RANGE);
          on = false;
        }
      }
      int bits = 0;
      if (on) {
        float ratio;
        sum += surrogate_term(logp[t], old_logp[t], A, cc, &bits, &ratio);
        ++cnt;
      }
      if (clip_mask) clip_mask[t] = static_cast<uint8_t>(bits);
    };
    for (int64_t u = (lo >> 2) + lane; (u << 2) < hi; u += LPR) {
      const int64_t t0 = u << 2;
      if (t0 + 4 <= L.n_tok) {
        // aligned 4-row vector; rows of a neighbouring response inside it are read but not used
        const float4 lp = *reinterpret_cast<const float4*>(logp + t0);
        const float4 ol = *reinterpret_cast<const float4*>(old_logp + t0);
        uint32_t m4 = 0x01010101u;
        if (L.mask) m4 = *reinterpret_cast<const uint32_t*>(L.mask + t0);
        int4 y4 = make_int4(0, 0, 0, 0);
        if (L.token_id) y4 = *reinterpret_cast<const int4*>(L.token_id + t0);
        const float lpv[4] = {lp.x, lp.y, lp.z, lp.w};
        const float olv[4] = {ol.x, ol.y, ol.z, ol.w};
        const int yv[4] = {y4.x, y4.y, y4.z, y4.w};
        const bool interior = (t0 >= lo) && (t0 + 4 <= hi);
        uint32_t out = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool mine = interior || (t0 + e >= lo && t0 + e < hi);
          bool on = mine && (head >= 0) && (((m4 >> (8 * e)) & 0xffu) != 0);
          if (on && L.token_id != nullptr && (yv[e] < 0 || yv[e] >= L.V)) {
            atomicOr(err, AT_GRPO_DATA_TOKEN_RANGE);
            on = false;
          }
          if (on) {
            int bits;
            float ratio;
            sum += surrogate_term(lpv[e], olv[e], A, cc, &bits, &ratio);
            ++cnt;
            out |= static_cast<uint32_t>(bits) << (8 * e);
          }
        }
        if (clip_mask) {
          if (interior) {
            *reinterpret_cast<uint32_t*>(clip_mask + t0) = out;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (t0 + e >= lo && t0 + e < hi) clip_mask[t0 + e] = static_cast<uint8_t>(out >> (8 * e));
          }
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (t0 + e >= lo && t0 + e < hi) one(t0 + e);
      }
    }
    // rows owned by no response (before the first / after the last range) carry no flags
    if (clip_mask && r == 0)
      for (int64_t t = lane; t < lo; t += LPR) clip_mask[t] = 0;
    if (clip_mask && r == L.n_resp - 1)
      for (int64_t t = hi + lane; t < L.n_tok; t += LPR) clip_mask[t] = 0;
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) {
      sum += __shfl_xor(sum, o, 64);
      cnt += __shfl_xor(cnt, o, 64);
    }
    if (lane == 0) {
      resp_sum[r] = (agg == AT_GRPO_AGG_SEQ_MEAN_TOKEN_MEAN && cnt > 0) ? sum / static_cast<float>(cnt) : sum;
      resp_cnt[r] = cnt;
      resp_head[r] = head;
    }
  }
}

// one 1024-thread block per head: fixed-order sums over the responses routed to it
__global__ __launch_bounds__(1024) void k_loss_final(int n_resp, const float* __restrict__ resp_sum,
                                                     const int32_t* __restrict__ resp_cnt,
                                                     const int32_t* __restrict__ resp_head, int agg,
                                                     float* __restrict__ loss, int32_t* __restrict__ n_valid) {
  __shared__ float fs[16];
  __shared__ int is[16], ir[16];
  const int m = blockIdx.x;
  float acc = 0.f;
  int cnt = 0, nresp = 0;
#pragma unroll 8
  for (int r = threadIdx.x; r < n_resp; r += 1024) {
    const bool mine = resp_head[r] == m;
    const float sv = resp_sum[r];
    const int cv = resp_cnt[r];
    acc += mine ? sv : 0.f;
    cnt += mine ? cv : 0;
    nresp += (mine && cv > 0) ? 1 : 0;
  }
  acc = wave_sum(acc);
  cnt = wave_sum_int(cnt);
  nresp = wave_sum_int(nresp);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
    fs[wave] = acc;
    is[wave] = cnt;
    ir[wave] = nresp;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    int c = 0, nr = 0;
    for (int w = 0; w < 16; ++w) {
      tot += fs[w];
      c += is[w];
      nr += ir[w];
    }
    const int denom = (agg == AT_GRPO_AGG_SEQ_MEAN_TOKEN_MEAN) ? nr : c;
    loss[m] = denom > 0 ? -tot / static_cast<float>(denom) : 0.f;
    if (n_valid) n_valid[m] = c;
  }
}

// Diagnostics of the clipped-ratio update, one wavefront per response: participating rows, rows below
// / above the clip range, rows on the clipped branch, and the sums of ratio - 1 - d and of the ratio.
struct DiagPartials {
  int32_t* head;    // [n_resp]
  int32_t* n;       // [n_resp] x 4: rows, low, high, zero-gradient (struct of arrays)
  int32_t* low;
  int32_t* high;
  int32_t* zero;
  float* kl;        // [n_resp]
  float* ratio;     // [n_resp]
};

__global__ __launch_bounds__(256) void k_diag_resp(TokenLayout L, const float* __restrict__ logp,
                                                   const float* __restrict__ old_logp,
                                                   const float* __restrict__ adv, ClipConst cc, DiagPartials P,
                                                   int32_t* __restrict__ err) {
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int n_waves = (gridDim.x * blockDim.x) >> 6;
  for (int r = wave; r < L.n_resp; r += n_waves) {
    const int64_t lo = L.cu_seqlens[r], hi = L.cu_seqlens[r + 1];
    int head = -1;
    int n = 0, low = 0, high = 0, zero = 0;
    float kl = 0.f, rs = 0.f;
    if (lo < 0 || hi < lo || hi > L.n_tok) {
      if (lane == 0) atomicOr(err, AT_GRPO_DATA_SEQLENS);
    } else {
      head = head_of_response(r, L.n_heads, L.n_agent, L.resp_agent, L.head_of_agent, err);
      const float A = adv[r];
      for (int64_t t = lo + lane; t < hi; t += 64) {
        bool on = (head >= 0) && (L.mask == nullptr || L.mask[t] != 0);
        if (on && L.token_id != nullptr) {
          const int y = L.token_id[t];
          if (y < 0 || y >= L.V) {
            atomicOr(err, AT_GRPO_DATA_TOKEN_RANGE);
            on = false;
          }
        }
        if (on) {
          const float d = logp[t] - old_logp[t];
          const bool is_low = d < cc.lo, is_high = d > cc.hi;
          ++n;
          low += is_low;
          high += is_high;
          zero += (is_high && A > 0.f) || (is_low && A < 0.f);
          kl += expm1f(d) - d;
          rs += expf(d);
        }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      n += __shfl_xor(n, o, 64);
      low += __shfl_xor(low, o, 64);
      high += __shfl_xor(high, o, 64);
      zero += __shfl_xor(zero, o, 64);
      kl += __shfl_xor(kl, o, 64);
      rs += __shfl_xor(rs, o, 64);
    }
    if (lane == 0) {
      P.head[r] = head;
      P.n[r] = n;
      P.low[r] = low;
      P.high[r] = high;
      P.zero[r] = zero;
      P.kl[r] = kl;
      P.ratio[r] = rs;
    }
  }
}

// one 1024-thread block per head: fixed-order sums of the per-response partials
__global__ __launch_bounds__(1024) void k_diag_final(int n_resp, DiagPartials P, int32_t* __restrict__ counts,
                                                     float* __restrict__ stats) {
  __shared__ int is[4][16];
  __shared__ float fs[2][16];
  const int m = blockIdx.x;
  int c[4] = {0, 0, 0, 0};
  float f[2] = {0.f, 0.f};
  for (int r = threadIdx.x; r < n_resp; r += 1024) {
    if (P.head[r] != m) continue;
    c[0] += P.n[r];
    c[1] += P.low[r];
    c[2] += P.high[r];
    c[3] += P.zero[r];
    f[0] += P.kl[r];
    f[1] += P.ratio[r];
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    c[k] = wave_sum_int(c[k]);
    if (lane == 0) is[k][wave] = c[k];
  }
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    f[k] = wave_sum(f[k]);
    if (lane == 0) fs[k][wave] = f[k];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot[4] = {0, 0, 0, 0};
    float ft[2] = {0.f, 0.f};
    for (int w = 0; w < 16; ++w) {
      for (int k = 0; k < 4; ++k) tot[k] += is[k][w];
      for (int k = 0; k < 2; ++k) ft[k] += fs[k][w];
    }
    for (int k = 0; k < 4; ++k) counts[m * 4 + k] = tot[k];
    stats[m * 2 + 0] = tot[0] > 0 ? ft[0] / static_cast<float>(tot[0]) : 0.f;
    stats[m * 2 + 1] = tot[0] > 0 ? ft[1] / static_cast<float>(tot[0]) : 0.f;
  }
}

__global__ __launch_bounds__(256) void k_coef(int64_t n_tok, int32_t* __restrict__ flag, CoefArgs ca,
                                              const float* __restrict__ logp, float* __restrict__ coef) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (t >= n_tok) return;
  const int f = flag[t];
  float g = 0.f;
  if (f >= 0) {
    g = coef_value(ca, f, t, logp[t]);
    if (g == 0.f) {
      g = 0.f;          // also folds -0
      flag[t] = -1;
    }
  }
  coef[t] = g;
}

__global__ __launch_bounds__(256) void k_split_by_advantage(int64_t n_tok, const int32_t* __restrict__ flag,
                                                            const int32_t* __restrict__ resp_of_tok,
                                                            const float* __restrict__ adv,
                                                            int32_t* __restrict__ flag_b,
                                                            int32_t* __restrict__ flag_f) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (t >= n_tok) return;
  const int f = flag[t];
  bool grad = false;
  if (f >= 0) grad = adv[resp_of_tok[t]] != 0.f;   // NaN counts as non-zero and propagates
  flag_b[t] = (f >= 0 && grad) ? f : -1;
  flag_f[t] = (f >= 0 && !grad) ? f : -1;
}

__global__ __launch_bounds__(256) void k_zero_nonparticipating(int64_t n_tok,
                                                               const int32_t* __restrict__ flag,
                                                               float* __restrict__ logp,
                                                               float* __restrict__ lse) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (t >= n_tok) return;
  if (flag[t] < 0) {
    logp[t] = 0.f;
    if (lse) lse[t] = 0.f;
  }
}

unsigned grid_for(int64_t n, int per_block, int64_t cap = 1 << 20) {
  int64_t g = ceil_div(n, per_block);
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return static_cast<unsigned>(g);
}

}  // namespace

int launch_fill_i32(int32_t* p, int64_t n, int32_t value, hipStream_t s) {
  if (n <= 0) return AT_GRPO_OK;
  hipLaunchKernelGGL(k_fill_i32, dim3(grid_for(n, 256, 4096)), dim3(256), 0, s, p, n, value);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_fill_bytes16(void* p, int64_t n_bytes, hipStream_t s) {
  if (n_bytes <= 0) return AT_GRPO_OK;
  ProfScope ps(PROF_FILL, s);
  hipLaunchKernelGGL(k_zero16, dim3(grid_for(n_bytes / 16, 256, 8192)), dim3(256), 0, s,
                     static_cast<uint4*>(p), n_bytes / 16);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_route(const TokenLayout& L, const TokenScratch& S, hipStream_t s) {
  ProfScope ps(PROF_PREP, s);
  ATG_TRY(launch_fill_i32(S.err, 1, 0, s));
  ATG_TRY(launch_fill_i32(S.resp_of_tok, L.n_tok, -1, s));
  ATG_TRY(launch_fill_i32(S.flag, L.n_tok, -1, s));
  hipLaunchKernelGGL(k_route, dim3(grid_for(L.n_resp, 4, 4096)), dim3(256), 0, s, L, S.err,
                     S.resp_of_tok, S.flag);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_compact(const TokenLayout& L, const TokenScratch& S, bool with_idx, hipStream_t s) {
  ProfScope ps(PROF_PREP, s);
  const unsigned nb = static_cast<unsigned>(S.n_blk);
  hipLaunchKernelGGL(k_count, dim3(nb), dim3(256), 0, s, S.flag, L.n_tok, L.n_heads, S.n_blk, S.blk_cnt);
  ATG_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(256), 0, s, S.blk_cnt, L.n_heads, S.n_blk, S.blk_off,
                     S.cnt);
  ATG_LAUNCH_CHECK();
  if (with_idx) {
    hipLaunchKernelGGL(k_scatter, dim3(nb), dim3(256), 0, s, S.flag, L.n_tok, L.n_heads, S.n_blk,
                       S.blk_off, S.idx);
    ATG_LAUNCH_CHECK();
  }
  return AT_GRPO_OK;
}

int launch_resp_len(const TokenLayout& L, const TokenScratch& S, hipStream_t s) {
  ProfScope ps(PROF_PREP, s);
  hipLaunchKernelGGL(k_resp_len, dim3(grid_for(L.n_resp, 4, 4096)), dim3(256), 0, s, L, S.flag,
                     S.resp_len);
  ATG_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_resp_cnt, dim3(1), dim3(256), 0, s, L, S.resp_len, S.err, S.resp_cnt);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_surrogate(const TokenLayout& L, const TokenScratch& S, const float* logp, const float* old_logp,
                     const float* adv, float eps_low, float eps_high, int agg, float* loss,
                     uint8_t* clip_mask, int32_t* n_valid, hipStream_t s) {
  ProfScope ps(PROF_SURROGATE, s);
  const ClipConst cc = make_clip(eps_low, eps_high);
  const int64_t mean_rows = L.n_tok / (L.n_resp > 0 ? L.n_resp : 1);
  if (mean_rows >= 512)
    hipLaunchKernelGGL(k_surrogate_resp<64>, dim3(grid_for(L.n_resp, 4, 16384)), dim3(256), 0, s, L, logp,
                       old_logp, adv, cc, agg, clip_mask, S.resp_sum, S.resp_len, S.resp_head, S.err);
  else if (mean_rows >= 160)
    hipLaunchKernelGGL(k_surrogate_resp<32>, dim3(grid_for(L.n_resp, 8, 16384)), dim3(256), 0, s, L, logp,
                       old_logp, adv, cc, agg, clip_mask, S.resp_sum, S.resp_len, S.resp_head, S.err);
  else
    hipLaunchKernelGGL(k_surrogate_resp<16>, dim3(grid_for(L.n_resp, 16, 16384)), dim3(256), 0, s, L, logp,
                       old_logp, adv, cc, agg, clip_mask, S.resp_sum, S.resp_len, S.resp_head, S.err);
  ATG_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_loss_final, dim3(L.n_heads), dim3(1024), 0, s, L.n_resp, S.resp_sum, S.resp_len,
                     S.resp_head, agg, loss, n_valid);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

size_t diagnostics_workspace(int32_t n_resp) {
  WsAlloc ws(nullptr);
  ws.take<int32_t>(64);
  for (int k = 0; k < 7; ++k) ws.take<int32_t>(static_cast<size_t>(n_resp));
  return ws.bytes();
}

int launch_diagnostics(const TokenLayout& L, const float* logp, const float* old_logp, const float* adv,
                       float eps_low, float eps_high, int32_t* counts, float* stats, void* workspace,
                       hipStream_t s) {
  ProfScope ps(PROF_SURROGATE, s);
  WsAlloc ws(workspace);
  int32_t* err = ws.take<int32_t>(64);
  DiagPartials P;
  P.head = ws.take<int32_t>(static_cast<size_t>(L.n_resp));
  P.n = ws.take<int32_t>(static_cast<size_t>(L.n_resp));
  P.low = ws.take<int32_t>(static_cast<size_t>(L.n_resp));
  P.high = ws.take<int32_t>(static_cast<size_t>(L.n_resp));
  P.zero = ws.take<int32_t>(static_cast<size_t>(L.n_resp));
  P.kl = reinterpret_cast<float*>(ws.take<int32_t>(static_cast<size_t>(L.n_resp)));
  P.ratio = reinterpret_cast<float*>(ws.take<int32_t>(static_cast<size_t>(L.n_resp)));
  ATG_TRY(launch_fill_i32(err, 1, 0, s));
  const ClipConst cc = make_clip(eps_low, eps_high);
  hipLaunchKernelGGL(k_diag_resp, dim3(grid_for(L.n_resp, 4, 16384)), dim3(256), 0, s, L, logp, old_logp, adv, cc,
                     P, err);
  ATG_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_diag_final, dim3(L.n_heads), dim3(1024), 0, s, L.n_resp, P, counts, stats);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

CoefArgs make_coef_args(const TokenScratch& S, const float* old_logp, const float* adv, float eps_low,
                        float eps_high, int agg, const float* grad_loss) {
  CoefArgs ca;
  ca.resp_of_tok = S.resp_of_tok;
  ca.resp_len = S.resp_len;
  ca.cnt = S.cnt;
  ca.resp_cnt = S.resp_cnt;
  ca.old_logp = old_logp;
  ca.adv = adv;
  ca.grad_loss = grad_loss;
  ca.cc = make_clip(eps_low, eps_high);
  ca.agg = agg;
  return ca;
}

int launch_coef(const TokenLayout& L, const TokenScratch& S, const float* logp, const float* old_logp,
                const float* adv, float eps_low, float eps_high, int agg, const float* grad_loss,
                float* coef, hipStream_t s) {
  ProfScope ps(PROF_COEF, s);
  const CoefArgs ca = make_coef_args(S, old_logp, adv, eps_low, eps_high, agg, grad_loss);
  hipLaunchKernelGGL(k_coef, dim3(static_cast<unsigned>(S.n_blk256)), dim3(256), 0, s, L.n_tok, S.flag, ca, logp,
                     coef);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_split_by_advantage(const TokenLayout& L, const TokenScratch& S, const float* adv, int32_t* flag_b,
                              int32_t* flag_f, hipStream_t s) {
  ProfScope ps(PROF_PREP, s);
  hipLaunchKernelGGL(k_split_by_advantage, dim3(static_cast<unsigned>(S.n_blk256)), dim3(256), 0, s, L.n_tok,
                     S.flag, S.resp_of_tok, adv, flag_b, flag_f);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

int launch_zero_nonparticipating(const TokenLayout& L, const TokenScratch& S, float* logp, float* lse,
                                 hipStream_t s) {
  ProfScope ps(PROF_PREP, s);
  hipLaunchKernelGGL(k_zero_nonparticipating, dim3(static_cast<unsigned>(S.n_blk256)), dim3(256), 0, s,
                     L.n_tok, S.flag, logp, lse);
  ATG_LAUNCH_CHECK();
  return AT_GRPO_OK;
}

}  // namespace atg
