// Launchers of the per-token streaming kernels: routing of rows to responses and heads, validity
// flags, stable per-head compaction, the clipped surrogate with its deterministic reduction, and
// the backward coefficient.
#pragma once

#include <math.h>

#include "common.hpp"

namespace atg {

constexpr int kTokPerBlock = 2048;   // tokens handled by one 256-thread block (8 per thread)

struct TokenLayout {
  int64_t n_tok;
  int32_t n_resp, n_heads, n_agent, V;
  const int64_t* cu_seqlens;
  const int32_t* token_id;
  const uint8_t* mask;
  const int32_t* resp_agent;
  const int32_t* head_of_agent;
};

struct TokenScratch {
  int32_t* err;          // [1] device error word
  int32_t* resp_of_tok;  // [n_tok]
  int32_t* flag;         // [n_tok] head of a participating row, -1 otherwise
  int32_t* blk_cnt;      // [n_heads * n_blk]
  int32_t* blk_off;      // [n_heads * n_blk]
  int32_t* cnt;          // [kMaxHeads] participating rows per head
  int32_t* idx;          // [n_heads * n_tok] compacted rows per head
  int32_t* resp_len;     // [n_resp] participating rows per response
  int32_t* resp_cnt;     // [kMaxHeads] responses with at least one participating row, per head
  float* resp_sum;       // [n_resp] per-response sum (or mean) of surrogate terms
  int32_t* resp_head;    // [n_resp] head of each response (-1: takes no part)
  int64_t n_blk;         // ceil(n_tok / kTokPerBlock)
  int64_t n_blk256;      // ceil(n_tok / 256)
};

// ---- Eq. (2) per token ---------------------------------------------------------------------------
struct ClipConst {
  float lo, hi;          // log-space thresholds
  float one_minus, one_plus;
};

inline ClipConst make_clip(float eps_low, float eps_high) {
  ClipConst c;
  c.lo = static_cast<float>(log1p(-static_cast<double>(eps_low)));
  c.hi = static_cast<float>(log1p(static_cast<double>(eps_high)));
  c.one_minus = 1.f - eps_low;
  c.one_plus = 1.f + eps_high;
  return c;
}

// What the backward coefficient of one row needs besides its log-probability.
struct CoefArgs {
  const int32_t* resp_of_tok;   // [n_tok]
  const int32_t* resp_len;      // [n_resp] participating rows per response (sequence-mean aggregation)
  const int32_t* cnt;           // [kMaxHeads] participating rows per head (token-mean aggregation)
  const int32_t* resp_cnt;      // [kMaxHeads] responses with a participating row, per head
  const float* old_logp;
  const float* adv;
  const float* grad_loss;       // [n_heads] or null (= 1)
  ClipConst cc;
  int agg;
};

CoefArgs make_coef_args(const TokenScratch& S, const float* old_logp, const float* adv, float eps_low,
                        float eps_high, int agg, const float* grad_loss);

#ifdef __HIPCC__
// Per-token pieces of Eq. (2).  Returns l_t; sets *bits and *ratio.
__device__ __forceinline__ float surrogate_term(float logp, float old_logp, float A, const ClipConst& c,
                                                int* bits, float* ratio) {
  const float d = logp - old_logp;
  const float r = expf(d);
  const bool low = d < c.lo, high = d > c.hi;
  const bool zero = (high && A > 0.f) || (low && A < 0.f);
  *bits = (low ? AT_GRPO_CLIP_LOW : 0) | (high ? AT_GRPO_CLIP_HIGH : 0) | (zero ? AT_GRPO_CLIP_ZERO_GRAD : 0);
  *ratio = r;
  return zero ? (high ? c.one_plus : c.one_minus) * A : r * A;
}

// g_t = d loss / d logp_t of a participating row t of head `head` (0 on the clipped branch).
__device__ __forceinline__ float coef_value(const CoefArgs& a, int head, int64_t t, float logp) {
  const int r = a.resp_of_tok[t];
  const float A = a.adv[r];
  int bits;
  float ratio;
  surrogate_term(logp, a.old_logp[t], A, a.cc, &bits, &ratio);
  float w;
  if (a.agg == AT_GRPO_AGG_SEQ_MEAN_TOKEN_MEAN)
    w = 1.f / (static_cast<float>(a.resp_cnt[head]) * static_cast<float>(a.resp_len[r]));
  else
    w = 1.f / static_cast<float>(a.cnt[head]);
  if (bits & AT_GRPO_CLIP_ZERO_GRAD) return 0.f;
  return -w * A * ratio * (a.grad_loss ? a.grad_loss[head] : 1.f);
}
#endif  // __HIPCC__

int launch_fill_i32(int32_t* p, int64_t n, int32_t value, hipStream_t s);
int launch_fill_bytes16(void* p, int64_t n_bytes, hipStream_t s);   // zero fill, n_bytes % 16 == 0

// resp_of_tok, flag (participation by mask / token range / routing), error word checks.
int launch_route(const TokenLayout& L, const TokenScratch& S, hipStream_t s);

// cnt[m] and, when with_idx, the stable compaction idx[m * n_tok + ...] of rows with flag == m.
int launch_compact(const TokenLayout& L, const TokenScratch& S, bool with_idx, hipStream_t s);

// resp_len / resp_cnt (only needed for the sequence-mean aggregation).
int launch_resp_len(const TokenLayout& L, const TokenScratch& S, hipStream_t s);

// Per-token surrogate terms + clip mask + per-head loss (Eq. 2).  Self-contained: reads the layout
// directly (one wavefront per response); overwrites resp_len with its own per-response counts.
int launch_surrogate(const TokenLayout& L, const TokenScratch& S, const float* logp,
                     const float* old_logp, const float* adv, float eps_low, float eps_high, int agg,
                     float* loss, uint8_t* clip_mask, int32_t* n_valid, hipStream_t s);

// Diagnostics of the clipped-ratio update: counts[n_heads][4] = (rows, below, above, zero-gradient),
// stats[n_heads][2] = (mean of ratio - 1 - d, mean ratio).  Self-contained like launch_surrogate; its
// scratch (an error word and seven per-response arrays) is taken from `workspace`.
size_t diagnostics_workspace(int32_t n_resp);
int launch_diagnostics(const TokenLayout& L, const float* logp, const float* old_logp, const float* adv,
                       float eps_low, float eps_high, int32_t* counts, float* stats, void* workspace,
                       hipStream_t s);

// Backward coefficient coef[t] = d loss / d logp_t; rewrites flag to -1 where coef == 0.
int launch_coef(const TokenLayout& L, const TokenScratch& S, const float* logp, const float* old_logp,
                const float* adv, float eps_low, float eps_high, int agg, const float* grad_loss,
                float* coef, hipStream_t s);

// Splits the participating rows by their response's advantage: flag_b = flag where adv != 0 (these rows can
// carry gradient), flag_f = flag where adv == 0 (log-probability only); -1 elsewhere in both.
int launch_split_by_advantage(const TokenLayout& L, const TokenScratch& S, const float* adv, int32_t* flag_b,
                              int32_t* flag_f, hipStream_t s);

// logp = lse = 0 on rows with flag < 0.
int launch_zero_nonparticipating(const TokenLayout& L, const TokenScratch& S, float* logp, float* lse,
                                 hipStream_t s);

}  // namespace atg
