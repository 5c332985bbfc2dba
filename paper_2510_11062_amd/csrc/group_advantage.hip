// Agent- and turn-wise grouping and group-relative advantages (gfx950).
//
// Alg. 1 of the paper keys every sampled candidate by g = hash(e, i, t); Eq. (1) normalises the
// rewards inside each group.  Here the key is the injective packing
//   key = (e * n_agent + i) * n_turn + t,
// groups are numbered densely in ascending key order, and the responses of a group are listed in
// ascending original index (a stable sort by key).  Pipeline: histogram over the key space ->
// exclusive scans (present keys -> dense ids, member counts -> CSR offsets) -> scatter by the
// arrival rank the histogram's atomic returned (arbitrary order) -> per-group ordering of the
// segment and the fp32 statistics.  The final ordering makes every output deterministic.
// Three launch shapes, same device functions: everything in one workgroup (small batches: one
// launch), five launches with a one-workgroup scan (key boxes up to 65536), seven launches with a
// three-kernel scan (anything larger).
#include <mutex>

#include "common.hpp"

namespace atg {

namespace {

constexpr int kKeysPerBlock = 2048;
constexpr int kSmallGroup = 16;

struct GaArgs {
  int32_t n_resp, n_env, n_agent, n_turn;
  const int32_t* env_id;
  const int32_t* agent_id;
  const int32_t* turn_id;
  const float* reward;
  int32_t group_by;          // at_grpo_group_by
  int32_t n_sample;          // extent of sample_id (AT_GRPO_GROUP_BY_PARALLEL only)
  const int32_t* sample_id;  // candidate index c of each response (AT_GRPO_GROUP_BY_PARALLEL only)
};

// Key of a response under the chosen grouping (ascending key = canonical group order):
//   AGENT_TURN  (e, i, t)                         the paper's grouping (Alg. 1, Sec. 4.1)
//   TRAJECTORY  e                                 all candidates of a task in one group, whatever agent
//                                                 and turn produced them (GRPO applied to the whole MAS)
//   PARALLEL    (e, i, t, c if t > 0 else 0)      K trajectories sampled in parallel share a state only at
//                                                 the first turn; later turns are groups of one (Sec. 4.1)
// A response with an id outside its extent has no key.
__device__ __forceinline__ int64_t key_of(const GaArgs& a, int r, bool* ok) {
  const int e = a.env_id[r], i = a.agent_id[r], t = a.turn_id[r];
  bool in = e >= 0 && e < a.n_env && i >= 0 && i < a.n_agent && t >= 0 && t < a.n_turn;
  int64_t key;
  if (a.group_by == AT_GRPO_GROUP_BY_TRAJECTORY) {
    key = e;
  } else {
    key = (static_cast<int64_t>(e) * a.n_agent + i) * a.n_turn + t;
    if (a.group_by == AT_GRPO_GROUP_BY_PARALLEL) {
      const int c = a.sample_id[r];
      in = in && c >= 0 && c < a.n_sample;
      key = key * a.n_sample + (t > 0 ? c : 0);
    }
  }
  *ok = in;
  return key;
}

__device__ __forceinline__ bool finite_reward(float x) { return fabsf(x) <= 3.402823466e38f; }

// Histogram over the key box.  The atomic's return value is the response's arrival rank inside its
// group.  Neighbouring lanes with the same key (candidates of one group emitted together, the
// order a rollout produces) are folded into one atomic per run.
__global__ __launch_bounds__(256) void k_ga_hist(GaArgs a, int32_t* __restrict__ err,
                                                 int32_t* __restrict__ hist, int32_t* __restrict__ key_of_resp,
                                                 int32_t* __restrict__ rank_of_resp) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  const int lane = threadIdx.x & 63;
  int key = -1;
  if (r < a.n_resp) {
    bool ok;
    const int64_t k64 = key_of(a, r, &ok);
    if (!ok) {
      atomicOr(err, AT_GRPO_DATA_ID_RANGE);
    } else if (!finite_reward(a.reward[r])) {
      atomicOr(err, AT_GRPO_DATA_REWARD);     // takes no part: no group, advantage 0
    } else {
      key = static_cast<int32_t>(k64);
    }
    key_of_resp[r] = key;
  }
  // runs of equal keys inside the wavefront
  const int prev = __shfl_up(key, 1, 64);
  const bool head = (lane == 0) || (key != prev);
  const unsigned long long heads = __builtin_amdgcn_ballot_w64(head);
  const unsigned long long below = heads & ((2ull << lane) - 1ull);          // heads at or below this lane
  const int start = 63 - __builtin_clzll(below);
  const unsigned long long above = (lane == 63) ? 0ull : (heads >> (lane + 1)) << (lane + 1);
  const int next = above ? __builtin_ctzll(above) : 64;
  int base = 0;
  if (head && key >= 0) base = atomicAdd(&hist[key], next - lane);
  base = __shfl(base, start, 64);
  if (r < a.n_resp && key >= 0) rank_of_resp[r] = base + (lane - start);
}

// per-block sums of (key present, members) over 2048 keys
__global__ __launch_bounds__(256) void k_ga_scan_partial(const int32_t* __restrict__ hist, int64_t n_keys,
                                                         int32_t* __restrict__ bsum_p,
                                                         int32_t* __restrict__ bsum_c) {
  __shared__ int lds4[4];
  const int64_t k0 = static_cast<int64_t>(blockIdx.x) * kKeysPerBlock + threadIdx.x * 8;
  int p = 0, c = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int h = (k0 + e < n_keys) ? hist[k0 + e] : 0;
    p += (h > 0);
    c += h;
  }
  const int tp = block_sum_256_int(p, lds4);
  const int tcn = block_sum_256_int(c, lds4);
  if (threadIdx.x == 0) {
    bsum_p[blockIdx.x] = tp;
    bsum_c[blockIdx.x] = tcn;
  }
}

// single block: exclusive scan of the block sums; totals -> n_groups and the closing CSR offset
__global__ __launch_bounds__(256) void k_ga_scan_top(int64_t n_blocks, int32_t* __restrict__ bsum_p,
                                                     int32_t* __restrict__ bsum_c,
                                                     int32_t* __restrict__ n_groups,
                                                     int32_t* __restrict__ seg_offsets) {
  __shared__ int lds4[4];
  int run_p = 0, run_c = 0;
  for (int64_t base = 0; base < n_blocks; base += 256) {
    const int64_t b = base + threadIdx.x;
    const int vp = (b < n_blocks) ? bsum_p[b] : 0;
    const int vc = (b < n_blocks) ? bsum_c[b] : 0;
    int tp, tcn;
    const int ep = block_exclusive_scan_256(vp, lds4, &tp);
    const int ec = block_exclusive_scan_256(vc, lds4, &tcn);
    if (b < n_blocks) {
      bsum_p[b] = run_p + ep;
      bsum_c[b] = run_c + ec;
    }
    run_p += tp;
    run_c += tcn;
  }
  if (threadIdx.x == 0) {
    *n_groups = run_p;
    seg_offsets[run_p] = run_c;
  }
}

// dense id of every present key and CSR offset of every group
__global__ __launch_bounds__(256) void k_ga_scan_apply(const int32_t* __restrict__ hist, int64_t n_keys,
                                                       const int32_t* __restrict__ boff_p,
                                                       const int32_t* __restrict__ boff_c,
                                                       int32_t* __restrict__ gid_of_key,
                                                       int32_t* __restrict__ seg_offsets) {
  __shared__ int lds4[4];
  const int64_t k0 = static_cast<int64_t>(blockIdx.x) * kKeysPerBlock + threadIdx.x * 8;
  int h[8];
  int p = 0, c = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    h[e] = (k0 + e < n_keys) ? hist[k0 + e] : 0;
    p += (h[e] > 0);
    c += h[e];
  }
  int tp, tcn;
  int gp = boff_p[blockIdx.x] + block_exclusive_scan_256(p, lds4, &tp);
  int gc = boff_c[blockIdx.x] + block_exclusive_scan_256(c, lds4, &tcn);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if (h[e] > 0) {
      gid_of_key[k0 + e] = gp;
      seg_offsets[gp] = gc;
      ++gp;
      gc += h[e];
    }
  }
}

__global__ __launch_bounds__(256) void k_ga_scatter(int n_resp, const int32_t* __restrict__ key_of_resp,
                                                    const int32_t* __restrict__ rank_of_resp,
                                                    const int32_t* __restrict__ gid_of_key,
                                                    const int32_t* __restrict__ seg_offsets,
                                                    int32_t* __restrict__ group_id,
                                                    int32_t* __restrict__ arrival,
                                                    float* __restrict__ adv) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= n_resp) return;
  const int key = key_of_resp[r];
  if (key < 0) {
    group_id[r] = -1;
    adv[r] = 0.f;
    return;
  }
  const int g = gid_of_key[key];
  group_id[r] = g;
  arrival[seg_offsets[g] + rank_of_resp[r]] = r;
}

struct GaStat {
  float eps_std;
  int ddof, norm;
};

// Eq. (1) for one group, sequential in perm order (fp32, two passes).
__device__ __forceinline__ void group_stats_seq(const int32_t* perm_seg, int n,
                                                const float* __restrict__ reward, const GaStat& st,
                                                float* __restrict__ adv, float* mean_out, float* std_out) {
  const float x0 = reward[perm_seg[0]];
  float sum = 0.f;
  bool same = true;
  for (int j = 0; j < n; ++j) {
    const float x = reward[perm_seg[j]];
    sum += x;
    same = same && (x == x0);
  }
  if (same) {
    for (int j = 0; j < n; ++j) adv[perm_seg[j]] = 0.f;
    *mean_out = x0;
    *std_out = 0.f;
    return;
  }
  const float mean = sum / static_cast<float>(n);
  float ss = 0.f;
  for (int j = 0; j < n; ++j) {
    const float d = reward[perm_seg[j]] - mean;
    ss += d * d;
  }
  const int denom = n - st.ddof;
  const float sd = denom > 0 ? sqrtf(ss / static_cast<float>(denom)) : 0.f;
  for (int j = 0; j < n; ++j) {
    const int r = perm_seg[j];
    adv[r] = (st.norm == AT_GRPO_NORM_STD) ? (reward[r] - mean) / (sd + st.eps_std) : (reward[r] - mean);
  }
  *mean_out = mean;
  *std_out = sd;
}

// One group of at most kSmallGroup members, handled by one thread: order the segment, Eq. (1).
__device__ __forceinline__ void finish_group_by_thread(int g, const int32_t* __restrict__ seg_offsets,
                                                       const int32_t* __restrict__ arrival,
                                                       const float* __restrict__ reward, const GaStat& st,
                                                       int32_t* perm, float* __restrict__ adv,
                                                       float* __restrict__ group_mean,
                                                       float* __restrict__ group_std) {
  const int off = seg_offsets[g], n = seg_offsets[g + 1] - off;
  if (n > kSmallGroup) return;
  if (n <= 8) {
    // whole group in registers: ranks by counting, sums taken in ascending-index order
    int id[8];
    float x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) id[j] = (j < n) ? arrival[off + j] : 0x7fffffff;
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = (j < n) ? reward[id[j]] : 0.f;
    int rank[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int c = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) c += (id[i] < id[j]);
      rank[j] = c;
    }
    float xs[8];      // rewards in perm order
#pragma unroll
    for (int pos = 0; pos < 8; ++pos) {
      float v = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) v = (rank[j] == pos && j < n) ? x[j] : v;
      xs[pos] = v;
    }
    float sum = 0.f;
    bool same = true;
#pragma unroll
    for (int pos = 0; pos < 8; ++pos)
      if (pos < n) {
        sum += xs[pos];
        same = same && (xs[pos] == xs[0]);
      }
    float mean = same ? xs[0] : sum / static_cast<float>(n), sd = 0.f, ss = 0.f;
#pragma unroll
    for (int pos = 0; pos < 8; ++pos)
      if (pos < n) {
        const float d = xs[pos] - mean;
        ss += d * d;
      }
    const int denom = n - st.ddof;
    if (!same) sd = denom > 0 ? sqrtf(ss / static_cast<float>(denom)) : 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < n) {
        perm[off + rank[j]] = id[j];
        float a = 0.f;
        if (!same) a = (st.norm == AT_GRPO_NORM_STD) ? (x[j] - mean) / (sd + st.eps_std) : (x[j] - mean);
        adv[id[j]] = a;
      }
    if (group_mean) group_mean[g] = mean;
    if (group_std) group_std[g] = sd;
    return;
  }
  for (int j = 0; j < n; ++j) {
    const int rj = arrival[off + j];
    int rank = 0;
    for (int i = 0; i < n; ++i) rank += (arrival[off + i] < rj);
    perm[off + rank] = rj;
  }
  // perm[off .. off+n) was written by this thread only
  float mu, sd;
  group_stats_seq(perm + off, n, reward, st, adv, &mu, &sd);
  if (group_mean) group_mean[g] = mu;
  if (group_std) group_std[g] = sd;
}

// One larger group, handled by one wavefront: ranks by counting, statistics combined in a fixed order.
__device__ __forceinline__ void finish_group_by_wave(int g, int lane, const int32_t* __restrict__ seg_offsets,
                                                     const int32_t* __restrict__ arrival,
                                                     const float* __restrict__ reward, const GaStat& st,
                                                     int32_t* perm, float* __restrict__ adv,
                                                     float* __restrict__ group_mean,
                                                     float* __restrict__ group_std) {
  const int off = seg_offsets[g], n = seg_offsets[g + 1] - off;
  if (n <= kSmallGroup) return;
  for (int j = lane; j < n; j += 64) {
    const int rj = arrival[off + j];
    int rank = 0;
    for (int i = 0; i < n; ++i) rank += (arrival[off + i] < rj);
    perm[off + rank] = rj;
  }
  __threadfence();   // the ranks below are read back by other lanes of this wavefront
  // statistics: lane-strided partial sums combined in a fixed order
  const float x0 = reward[perm[off]];
  float sum = 0.f;
  int same = 1;
  for (int j = lane; j < n; j += 64) {
    const float x = reward[perm[off + j]];
    sum += x;
    same &= (x == x0);
  }
  sum = wave_sum(sum);
  sum = __shfl(sum, 0, 64);
  same = __builtin_amdgcn_ballot_w64(same == 0) == 0ull;
  float mean = sum / static_cast<float>(n), sd = 0.f;
  if (same) {
    for (int j = lane; j < n; j += 64) adv[perm[off + j]] = 0.f;
    mean = x0;
  } else {
    float ss = 0.f;
    for (int j = lane; j < n; j += 64) {
      const float d = reward[perm[off + j]] - mean;
      ss += d * d;
    }
    ss = wave_sum(ss);
    ss = __shfl(ss, 0, 64);
    const int denom = n - st.ddof;
    sd = denom > 0 ? sqrtf(ss / static_cast<float>(denom)) : 0.f;
    for (int j = lane; j < n; j += 64) {
      const int r = perm[off + j];
      adv[r] = (st.norm == AT_GRPO_NORM_STD) ? (reward[r] - mean) / (sd + st.eps_std) : (reward[r] - mean);
    }
  }
  if (lane == 0) {
    if (group_mean) group_mean[g] = mean;
    if (group_std) group_std[g] = sd;
  }
}

// Eq. (3): r = alpha * r_team + r_loc.  One fp32 multiplication, then one fp32 addition (never
// contracted to an fma): the result decides which groups count as all-equal and which candidate
// is the arg max, so its rounding is part of the definition.
__global__ __launch_bounds__(256) void k_ga_mix(int n, const float* __restrict__ r_team,
                                                const float* __restrict__ r_loc, float alpha,
                                                float* __restrict__ reward) {
#pragma clang fp contract(off)
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r < n) {
    const float prod = alpha * r_team[r];
    reward[r] = prod + r_loc[r];
  }
}

// Tree-structured sampling (Alg. 1): c* = arg max_c r^(c) per group, the first of equal rewards.
// perm lists a group's members in ascending response index, so a strict comparison keeps the first.
__global__ __launch_bounds__(256) void k_ga_select(const int32_t* __restrict__ n_groups,
                                                   const int32_t* __restrict__ seg_offsets,
                                                   const int32_t* __restrict__ perm,
                                                   const float* __restrict__ reward,
                                                   int32_t* __restrict__ best) {
  const int G = *n_groups;
  const int stride = gridDim.x * 256;
  for (int g = blockIdx.x * 256 + threadIdx.x; g < G; g += stride) {
    const int off = seg_offsets[g], n = seg_offsets[g + 1] - off;
    int top = perm[off];
    float xt = reward[top];
    for (int j = 1; j < n; ++j) {
      const int r = perm[off + j];
      const float x = reward[r];
      if (x > xt) {
        xt = x;
        top = r;
      }
    }
    best[g] = top;
  }
}

// ------------------------------------------------------------------------------------------------
// The whole call in one workgroup, for the sizes a training step actually has (a few thousand
// groups, a few ten thousand responses): histogram, scans and the key tables live in LDS and the
// phases are separated by workgroup barriers instead of kernel boundaries, so the call costs one
// launch instead of five or seven.  Same arithmetic and the same device functions as the multi-launch path.
// ------------------------------------------------------------------------------------------------
constexpr int kSingleThreads = 1024;
constexpr int kSingleMaxKeys = 8192;     // 3 tables of this many ints in LDS (96 KiB)
constexpr int kSingleMaxResp = 4096;     // beyond this the multi-launch path is faster

struct GaMix {
  const float* r_team;
  const float* r_loc;
  float alpha;
  float* reward_out;
};

// exclusive scan of one int per thread over the 1024-thread workgroup; *total = sum
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
  int base = 0, sum = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    const int t = lds16[w];
    if (w < wave) base += t;
    sum += t;
  }
  *total = sum;
  return base + incl - v;
}

__global__ __launch_bounds__(kSingleThreads) void k_ga_single(
    GaArgs a, GaMix mix, GaStat st, int n_keys, int32_t* __restrict__ err, int32_t* __restrict__ key_of_resp,
    int32_t* __restrict__ rank_of_resp, int32_t* __restrict__ arrival, int32_t* __restrict__ group_id,
    int32_t* __restrict__ n_groups, int32_t* __restrict__ seg_offsets, int32_t* perm,
    float* __restrict__ adv, float* __restrict__ group_mean, float* __restrict__ group_std,
    int32_t* __restrict__ best) {
  __shared__ int hist[kSingleMaxKeys];
  __shared__ int gid_of_key[kSingleMaxKeys];
  __shared__ int off_of_key[kSingleMaxKeys];
  __shared__ int lds16[16];
  __shared__ int s_groups;
  const int tid = threadIdx.x;
  if (tid == 0) *err = 0;
  for (int k = tid; k < n_keys; k += kSingleThreads) hist[k] = 0;
  if (mix.r_team) {
#pragma clang fp contract(off)
    for (int r = tid; r < a.n_resp; r += kSingleThreads) {
      const float prod = mix.alpha * mix.r_team[r];
      mix.reward_out[r] = prod + mix.r_loc[r];      // read back below by the thread that wrote it
    }
  }
  __syncthreads();

  // histogram: the atomic's return value is the arrival rank inside the group
  for (int r = tid; r < a.n_resp; r += kSingleThreads) {
    bool ok;
    const int64_t k64 = key_of(a, r, &ok);
    int key = -1;
    if (!ok) {
      atomicOr(err, AT_GRPO_DATA_ID_RANGE);
    } else if (!finite_reward(a.reward[r])) {
      atomicOr(err, AT_GRPO_DATA_REWARD);     // takes no part: no group, advantage 0
    } else {
      key = static_cast<int>(k64);
      rank_of_resp[r] = atomicAdd(&hist[key], 1);
    }
    key_of_resp[r] = key;
  }
  __syncthreads();

  // scans over the key box: present keys -> dense ids, member counts -> CSR offsets
  const int per = (n_keys + kSingleThreads - 1) / kSingleThreads;     // <= 8
  const int k0 = tid * per;
  int p = 0, c = 0;
  for (int e = 0; e < per; ++e) {
    const int h = (k0 + e < n_keys) ? hist[k0 + e] : 0;
    p += (h > 0);
    c += h;
  }
  int tot_p, tot_c;
  int gp = block_exclusive_scan_1024(p, lds16, &tot_p);
  int gc = block_exclusive_scan_1024(c, lds16, &tot_c);
  for (int e = 0; e < per; ++e) {
    const int h = (k0 + e < n_keys) ? hist[k0 + e] : 0;
    if (h > 0) {
      gid_of_key[k0 + e] = gp;
      off_of_key[k0 + e] = gc;
      seg_offsets[gp] = gc;
      ++gp;
      gc += h;
    }
  }
  if (tid == 0) {
    *n_groups = tot_p;
    seg_offsets[tot_p] = tot_c;
    s_groups = tot_p;
  }
  __syncthreads();

  // scatter by arrival rank
  for (int r = tid; r < a.n_resp; r += kSingleThreads) {
    const int key = key_of_resp[r];
    if (key < 0) {
      group_id[r] = -1;
      adv[r] = 0.f;
      continue;
    }
    group_id[r] = gid_of_key[key];
    arrival[off_of_key[key] + rank_of_resp[r]] = r;
  }
  __syncthreads();   // arrival and seg_offsets (global) are read by other threads below

  const int G = s_groups;
  for (int g = tid; g < G; g += kSingleThreads)
    finish_group_by_thread(g, seg_offsets, arrival, a.reward, st, perm, adv, group_mean, group_std);
  const int lane = tid & 63, wave = tid >> 6;
  for (int g = wave; g < G; g += kSingleThreads / 64)
    finish_group_by_wave(g, lane, seg_offsets, arrival, a.reward, st, perm, adv, group_mean, group_std);
  if (best) {
    __syncthreads();   // perm is complete
    for (int g = tid; g < G; g += kSingleThreads) {
      const int off = seg_offsets[g], n = seg_offsets[g + 1] - off;
      int top = perm[off];
      float xt = a.reward[top];
      for (int j = 1; j < n; ++j) {
        const int r = perm[off + j];
        const float x = a.reward[r];
        if (x > xt) {
          xt = x;
          top = r;
        }
      }
      best[g] = top;
    }
  }
}

// both finishing roles in one launch: the first n_small blocks take the small groups (a thread each),
// the remaining blocks the larger ones (a wavefront each)
__global__ __launch_bounds__(256) void k_ga_finish(int n_small, const int32_t* __restrict__ n_groups,
                                                   const int32_t* __restrict__ seg_offsets,
                                                   const int32_t* __restrict__ arrival,
                                                   const float* __restrict__ reward, GaStat st, int32_t* perm,
                                                   float* __restrict__ adv, float* __restrict__ group_mean,
                                                   float* __restrict__ group_std) {
  const int G = *n_groups;
  if (static_cast<int>(blockIdx.x) < n_small) {
    const int stride = n_small * 256;
    for (int g = blockIdx.x * 256 + threadIdx.x; g < G; g += stride)
      finish_group_by_thread(g, seg_offsets, arrival, reward, st, perm, adv, group_mean, group_std);
  } else {
    const int lane = threadIdx.x & 63;
    const int wave = ((blockIdx.x - n_small) * 256 + threadIdx.x) >> 6;
    const int n_waves = ((gridDim.x - n_small) * 256) >> 6;
    for (int g = wave; g < G; g += n_waves)
      finish_group_by_wave(g, lane, seg_offsets, arrival, reward, st, perm, adv, group_mean, group_std);
  }
}

// both scans over a key box of at most kScanSingleKeys keys in one workgroup
constexpr int kScanSingleKeys = 65536;
__global__ __launch_bounds__(kSingleThreads) void k_ga_scan_single(const int32_t* __restrict__ hist, int n_keys,
                                                                   int32_t* __restrict__ gid_of_key,
                                                                   int32_t* __restrict__ n_groups,
                                                                   int32_t* __restrict__ seg_offsets) {
  __shared__ int lds16[16];
  const int per = (n_keys + kSingleThreads - 1) / kSingleThreads;
  const int k0 = threadIdx.x * per;
  int p = 0, c = 0;
  for (int e = 0; e < per; ++e) {
    const int h = (k0 + e < n_keys) ? hist[k0 + e] : 0;
    p += (h > 0);
    c += h;
  }
  int tot_p, tot_c;
  int gp = block_exclusive_scan_1024(p, lds16, &tot_p);
  int gc = block_exclusive_scan_1024(c, lds16, &tot_c);
  for (int e = 0; e < per; ++e) {
    const int h = (k0 + e < n_keys) ? hist[k0 + e] : 0;
    if (h > 0) {
      gid_of_key[k0 + e] = gp;
      seg_offsets[gp] = gc;
      ++gp;
      gc += h;
    }
  }
  if (threadIdx.x == 0) {
    *n_groups = tot_p;
    seg_offsets[tot_p] = tot_c;
  }
}

// clears two ranges in one launch
__global__ void k_ga_clear2(int32_t* __restrict__ p, int64_t n, int32_t* __restrict__ q, int64_t nq) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < nq; i += stride) q[i] = 0;
}

struct GaPlan {
  int64_t n_keys, n_blocks;
  int32_t *err, *hist, *gid_of_key, *key_of_resp, *rank_of_resp, *arrival, *bsum_p, *bsum_c;
};

int64_t key_box(int32_t n_env, int32_t n_agent, int32_t n_turn, int32_t group_by, int32_t n_sample) {
  if (group_by == AT_GRPO_GROUP_BY_TRAJECTORY) return n_env;
  const int64_t eit = static_cast<int64_t>(n_env) * n_agent * n_turn;
  if (group_by == AT_GRPO_GROUP_BY_PARALLEL) return n_sample > 0 && eit <= (int64_t{1} << 28) ? eit * n_sample : -1;
  return eit;
}

bool plan(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn, int32_t group_by, int32_t n_sample,
          WsAlloc& ws, GaPlan* p) {
  if (n_resp <= 0 || n_env <= 0 || n_agent <= 0 || n_turn <= 0) return false;
  const int64_t n_keys = key_box(n_env, n_agent, n_turn, group_by, n_sample);
  if (n_keys <= 0 || n_keys > (int64_t{1} << 28)) return false;
  p->n_keys = n_keys;
  p->n_blocks = ceil_div(n_keys, kKeysPerBlock);
  p->err = ws.take<int32_t>(64);
  p->hist = ws.take<int32_t>(static_cast<size_t>(n_keys));
  p->gid_of_key = ws.take<int32_t>(static_cast<size_t>(n_keys));
  p->key_of_resp = ws.take<int32_t>(static_cast<size_t>(n_resp));
  p->rank_of_resp = ws.take<int32_t>(static_cast<size_t>(n_resp));
  p->arrival = ws.take<int32_t>(static_cast<size_t>(n_resp));
  p->bsum_p = ws.take<int32_t>(static_cast<size_t>(p->n_blocks));
  p->bsum_c = ws.take<int32_t>(static_cast<size_t>(p->n_blocks));
  return true;
}

}  // namespace

size_t group_advantage_workspace(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn, int32_t group_by,
                                 int32_t n_sample) {
  WsAlloc ws(nullptr);
  GaPlan p;
  if (!plan(n_resp, n_env, n_agent, n_turn, group_by, n_sample, ws, &p)) return 0;
  return ws.bytes();
}

size_t group_advantage_workspace(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn) {
  return group_advantage_workspace(n_resp, n_env, n_agent, n_turn, AT_GRPO_GROUP_BY_AGENT_TURN, 1);
}

}  // namespace atg

using namespace atg;

namespace {

int run_group_advantage(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn,
                        const int32_t* env_id, const int32_t* agent_id, const int32_t* turn_id,
                        const float* reward, float eps_std, int32_t ddof, int32_t norm, int32_t* group_id,
                        int32_t* n_groups, int32_t* seg_offsets, int32_t* perm, float* adv,
                        float* group_mean, float* group_std, const float* r_team, const float* r_loc,
                        float alpha, float* reward_out, int32_t* best, void* workspace,
                        size_t workspace_bytes, void* hip_stream,
                        int32_t group_by = AT_GRPO_GROUP_BY_AGENT_TURN, const int32_t* sample_id = nullptr,
                        int32_t n_sample = 1) {
  if (!env_id || !agent_id || !turn_id || !group_id || !n_groups || !seg_offsets || !perm || !adv)
    return AT_GRPO_EINVAL;
  if (n_resp <= 0 || n_env <= 0 || n_agent <= 0 || n_turn <= 0) return AT_GRPO_EINVAL;
  if (group_by != AT_GRPO_GROUP_BY_AGENT_TURN && group_by != AT_GRPO_GROUP_BY_TRAJECTORY &&
      group_by != AT_GRPO_GROUP_BY_PARALLEL)
    return AT_GRPO_EINVAL;
  if (group_by == AT_GRPO_GROUP_BY_PARALLEL && (!sample_id || n_sample <= 0)) return AT_GRPO_EINVAL;
  if (ddof != 0 && ddof != 1) return AT_GRPO_EINVAL;
  if (norm != AT_GRPO_NORM_STD && norm != AT_GRPO_NORM_NONE) return AT_GRPO_EINVAL;
  if (!(eps_std >= 0.f)) return AT_GRPO_EINVAL;
  WsAlloc ws(workspace);
  GaPlan p;
  if (!plan(n_resp, n_env, n_agent, n_turn, group_by, n_sample, ws, &p)) return AT_GRPO_EUNSUPPORTED;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < ws.bytes())
    return AT_GRPO_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  ProfScope ps(PROF_GROUP, s);

  if (p.n_keys <= kSingleMaxKeys && n_resp <= kSingleMaxResp) {
    const GaMix mix{r_team, r_loc, alpha, reward_out};
    const GaArgs a1{n_resp, n_env, n_agent, n_turn, env_id, agent_id, turn_id, r_team ? reward_out : reward,
                    group_by, n_sample, sample_id};
    const GaStat st1{eps_std, ddof, norm};
    hipLaunchKernelGGL(k_ga_single, dim3(1), dim3(kSingleThreads), 0, s, a1, mix, st1, static_cast<int>(p.n_keys),
                       p.err, p.key_of_resp, p.rank_of_resp, p.arrival, group_id, n_groups, seg_offsets, perm, adv,
                       group_mean, group_std, best);
    ATG_LAUNCH_CHECK();
    return AT_GRPO_OK;
  }
  if (r_team) {
    // the mixed reward is an output; everything below reads it
    hipLaunchKernelGGL(k_ga_mix, dim3(static_cast<unsigned>(ceil_div(n_resp, 256))), dim3(256), 0, s, n_resp,
                       r_team, r_loc, alpha, reward_out);
    ATG_LAUNCH_CHECK();
    reward = reward_out;
  }
  const GaArgs a{n_resp, n_env, n_agent, n_turn, env_id, agent_id, turn_id, reward, group_by, n_sample, sample_id};
  const GaStat st{eps_std, ddof, norm};
  const unsigned rb = static_cast<unsigned>(ceil_div(n_resp, 256));
  const unsigned kb = static_cast<unsigned>(p.n_blocks);

  hipLaunchKernelGGL(k_ga_clear2, dim3(static_cast<unsigned>(ceil_div(p.n_keys, 1024) > 4096 ? 4096 : ceil_div(p.n_keys, 1024))),
                     dim3(256), 0, s, p.hist, p.n_keys, p.err, int64_t{64});
  ATG_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_ga_hist, dim3(rb), dim3(256), 0, s, a, p.err, p.hist, p.key_of_resp, p.rank_of_resp);
  ATG_LAUNCH_CHECK();
  if (p.n_keys <= kScanSingleKeys) {
    hipLaunchKernelGGL(k_ga_scan_single, dim3(1), dim3(kSingleThreads), 0, s, p.hist, static_cast<int>(p.n_keys),
                       p.gid_of_key, n_groups, seg_offsets);
    ATG_LAUNCH_CHECK();
  } else {
    hipLaunchKernelGGL(k_ga_scan_partial, dim3(kb), dim3(256), 0, s, p.hist, p.n_keys, p.bsum_p, p.bsum_c);
    ATG_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_ga_scan_top, dim3(1), dim3(256), 0, s, p.n_blocks, p.bsum_p, p.bsum_c, n_groups,
                       seg_offsets);
    ATG_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_ga_scan_apply, dim3(kb), dim3(256), 0, s, p.hist, p.n_keys, p.bsum_p, p.bsum_c,
                       p.gid_of_key, seg_offsets);
    ATG_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(k_ga_scatter, dim3(rb), dim3(256), 0, s, n_resp, p.key_of_resp, p.rank_of_resp,
                     p.gid_of_key, seg_offsets, group_id, p.arrival, adv);
  ATG_LAUNCH_CHECK();
  // at most min(R, keys) groups exist; both finishing roles stride over them
  const int64_t g_max = n_resp < p.n_keys ? n_resp : p.n_keys;
  const unsigned fs = static_cast<unsigned>(ceil_div(g_max, 256) > 4096 ? 4096 : ceil_div(g_max, 256));
  const unsigned fl = static_cast<unsigned>(ceil_div(g_max, 4) > 4096 ? 4096 : ceil_div(g_max, 4));
  hipLaunchKernelGGL(k_ga_finish, dim3(fs + fl), dim3(256), 0, s, static_cast<int>(fs), n_groups, seg_offsets,
                     p.arrival, reward, st, perm, adv, group_mean, group_std);
  ATG_LAUNCH_CHECK();
  if (best) {
    hipLaunchKernelGGL(k_ga_select, dim3(fs), dim3(256), 0, s, n_groups, seg_offsets, perm, reward, best);
    ATG_LAUNCH_CHECK();
  }
  return AT_GRPO_OK;
}

}  // namespace

extern "C" int at_grpo_group_advantage(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn,
                                       const int32_t* env_id, const int32_t* agent_id,
                                       const int32_t* turn_id, const float* reward, float eps_std,
                                       int32_t ddof, int32_t norm, int32_t* group_id, int32_t* n_groups,
                                       int32_t* seg_offsets, int32_t* perm, float* adv, float* group_mean,
                                       float* group_std, void* workspace, size_t workspace_bytes,
                                       void* hip_stream) {
  if (!reward) return AT_GRPO_EINVAL;
  return run_group_advantage(n_resp, n_env, n_agent, n_turn, env_id, agent_id, turn_id, reward, eps_std, ddof,
                             norm, group_id, n_groups, seg_offsets, perm, adv, group_mean, group_std, nullptr,
                             nullptr, 0.f, nullptr, nullptr, workspace, workspace_bytes, hip_stream);
}

extern "C" int at_grpo_group_advantage_mixed(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn,
                                             const int32_t* env_id, const int32_t* agent_id,
                                             const int32_t* turn_id, const float* r_team,
                                             const float* r_loc, float alpha, float eps_std, int32_t ddof,
                                             int32_t norm, float* reward, int32_t* group_id,
                                             int32_t* n_groups, int32_t* seg_offsets, int32_t* perm,
                                             float* adv, float* group_mean, float* group_std,
                                             int32_t* best, void* workspace, size_t workspace_bytes,
                                             void* hip_stream) {
  if (!r_team || !r_loc || !reward) return AT_GRPO_EINVAL;
  if (!(fabsf(alpha) <= 3.402823466e38f)) return AT_GRPO_EINVAL;
  return run_group_advantage(n_resp, n_env, n_agent, n_turn, env_id, agent_id, turn_id, reward, eps_std, ddof,
                             norm, group_id, n_groups, seg_offsets, perm, adv, group_mean, group_std, r_team,
                             r_loc, alpha, reward, best, workspace, workspace_bytes, hip_stream);
}


extern "C" int at_grpo_group_advantage_keyed(int32_t group_by, int32_t n_resp, int32_t n_env, int32_t n_agent,
                                             int32_t n_turn, int32_t n_sample, const int32_t* env_id,
                                             const int32_t* agent_id, const int32_t* turn_id,
                                             const int32_t* sample_id, const float* reward, float eps_std,
                                             int32_t ddof, int32_t norm, int32_t* group_id, int32_t* n_groups,
                                             int32_t* seg_offsets, int32_t* perm, float* adv, float* group_mean,
                                             float* group_std, void* workspace, size_t workspace_bytes,
                                             void* hip_stream) {
  if (!reward) return AT_GRPO_EINVAL;
  return run_group_advantage(n_resp, n_env, n_agent, n_turn, env_id, agent_id, turn_id, reward, eps_std, ddof,
                             norm, group_id, n_groups, seg_offsets, perm, adv, group_mean, group_std, nullptr,
                             nullptr, 0.f, nullptr, nullptr, workspace, workspace_bytes, hip_stream, group_by,
                             sample_id, n_sample);
}

extern "C" size_t at_grpo_group_advantage_keyed_workspace_bytes(int32_t group_by, int32_t n_resp, int32_t n_env,
                                                                int32_t n_agent, int32_t n_turn, int32_t n_sample) {
  if (group_by != AT_GRPO_GROUP_BY_AGENT_TURN && group_by != AT_GRPO_GROUP_BY_TRAJECTORY &&
      group_by != AT_GRPO_GROUP_BY_PARALLEL)
    return 0;
  return group_advantage_workspace(n_resp, n_env, n_agent, n_turn, group_by, n_sample);
}

// ------------------------------------------------------------------------------------------------
// The same call for callers that cannot allocate or hand over device scratch: the workspace is a
// fixed array in device memory that belongs to the library.  Every GPU the library runs on holds
// its own copy of the array (at its own address) until the process ends.
// ------------------------------------------------------------------------------------------------
namespace {

constexpr size_t kStaticScratchBytes = size_t{2} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (looked up once per device; the array's name
// is only a host-side handle and must never be passed to a kernel or a memory call).
int static_scratch(void** out) {
  int dev = -1;
  ATG_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return AT_GRPO_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    ATG_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255)) return AT_GRPO_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return AT_GRPO_OK;
}

__global__ void k_ga_copy_error(const int32_t* __restrict__ err, int32_t* __restrict__ out) { *out = *err; }

}  // namespace

extern "C" size_t at_grpo_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int at_grpo_group_advantage_static(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn,
                                              const int32_t* env_id, const int32_t* agent_id,
                                              const int32_t* turn_id, const float* reward, float eps_std,
                                              int32_t ddof, int32_t norm, int32_t* group_id,
                                              int32_t* n_groups, int32_t* seg_offsets, int32_t* perm,
                                              float* adv, float* group_mean, float* group_std,
                                              int32_t* data_error, void* hip_stream) {
  if (!reward) return AT_GRPO_EINVAL;
  if (n_resp <= 0 || n_env <= 0 || n_agent <= 0 || n_turn <= 0) return AT_GRPO_EINVAL;
  const size_t need = group_advantage_workspace(n_resp, n_env, n_agent, n_turn);
  if (need == 0 || need > kStaticScratchBytes) return AT_GRPO_ESCRATCH;
  void* ws = nullptr;
  ATG_TRY(static_scratch(&ws));
  ATG_TRY(run_group_advantage(n_resp, n_env, n_agent, n_turn, env_id, agent_id, turn_id, reward, eps_std, ddof,
                              norm, group_id, n_groups, seg_offsets, perm, adv, group_mean, group_std, nullptr,
                              nullptr, 0.f, nullptr, nullptr, ws, kStaticScratchBytes, hip_stream));
  if (data_error) {
    hipLaunchKernelGGL(k_ga_copy_error, dim3(1), dim3(1), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const int32_t*>(ws), data_error);
    ATG_LAUNCH_CHECK();
  }
  return AT_GRPO_OK;
}
