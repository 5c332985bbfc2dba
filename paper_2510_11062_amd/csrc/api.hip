// C ABI entry points of the AT-GRPO policy-loss library: argument checks, workspace planning and
// the order in which the kernels are enqueued.  No call synchronises with the host.
#include <vector>

#include "common.hpp"
#include "head_kernels.hpp"
#include "token_kernels.hpp"

namespace atg {

size_t group_advantage_workspace(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn);
size_t head_update_workspace();

// ---- timing aid --------------------------------------------------------------------------------
namespace {
struct ProfState {
  bool on = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev[PROF_N];
};
ProfState g_prof;
const char* const kProfNames[PROF_N] = {"group_advantage", "token_prep", "head_fwd", "lse_combine",
                                        "surrogate", "coef", "transpose", "head_dz", "head_dh",
                                        "head_dw", "fill", "grad_norm", "adam", "head_fe"};
}  // namespace

void prof_begin(int cls, hipStream_t s) {
  if (!g_prof.on) return;
  hipEvent_t a = nullptr, b = nullptr;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
  (void)hipEventRecord(a, s);
  g_prof.ev[cls].emplace_back(a, b);
}

void prof_end(int cls, hipStream_t s) {
  if (!g_prof.on || g_prof.ev[cls].empty()) return;
  (void)hipEventRecord(g_prof.ev[cls].back().second, s);
}

int device_cu_count() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    cached[dev] = v;
  }
  return cached[dev];
}

namespace {

// Token rows per launch.  The token contraction (dW) reads and rewrites all of dW once per launch, so it
// takes the largest chunk the dZ buffer allows; the kernels that stream the hidden rows of the chunk once
// per band of vocabulary tiles (forward, dZ, dHidden) run faster on a part of it, whose hidden rows (64 MB)
// stay in the last-level cache beside the dZ rows being written (measured per step: H = 2048, 1 head:
// forward 155 -> 151 ms, dZ 156 -> 146 ms with 16384 rows, both slower again with 8192; H = 4096, 2 heads:
// dZ 1127 -> 1172 TFLOP/s with 8192 rows, forward 1163 -> 1305 TFLOP/s with 16384).
constexpr int kMaxChunkTokens = 32768;
constexpr int kSubChunkTokens = 16384;                 // forward launches; upper bound of the backward's sub-chunks
constexpr size_t kSubChunkBytes = size_t{64} << 20;    // hidden rows per dZ / dHidden launch: 16384 at H = 2048, 8192 at H = 4096
constexpr size_t kDzBudgetBytes = size_t{10} << 30;   // per orientation

struct Plan {
  TokenLayout L;
  TokenScratch S;
  HeadGeom g;
  int n_chunks;      // super-chunks per head in the worst case (all rows on one head)
  int sub;           // rows per launch of the dZ and dHidden kernels inside a super-chunk (divides g.TC)
  float* part_m;
  float* part_s;
  float* part_u;     // entropy call only
  float* zy;
  float* coef;
  void* Wt;
  void* hT;
  void* dZ;
  void* dZt;
  // one-pass forward + backward only
  TokenScratch SB, SF;   // the rows that can carry gradient / the rows with a zero advantage (own flag, cnt, idx)
  HeadGeom gF;           // geometry of the log-probability-only launches
  float* c2;             // [sub] reference of the exponentials
  float* scale;          // [TC] row factors of the super-chunk
  int32_t* gates;        // one word per launch of the exponentials
  int n_gates;
  int32_t* perm;         // [TC] list position of the row that sits at each place after the compaction
  int32_t* holes;        // [TC] scratch of the compaction
  int32_t* movers;       // [TC]
  int32_t* live_cnt;     // [0] rows with a non-zero factor, [1] rows moved
};

int check_layout(const at_grpo_batch* b, bool need_tensors) {
  if (!b) return AT_GRPO_EINVAL;
  if (b->n_tok <= 0 || b->n_resp <= 0 || b->V <= 0) return AT_GRPO_EINVAL;
  if (b->n_heads < 1 || b->n_heads > kMaxHeads) return AT_GRPO_EINVAL;
  if (b->n_tok > int64_t{0x7fffff00}) return AT_GRPO_EUNSUPPORTED;
  if (need_tensors) {
    if (b->dtype != AT_GRPO_F32 && b->dtype != AT_GRPO_BF16) return AT_GRPO_EUNSUPPORTED;
    if (b->H <= 0) return AT_GRPO_EINVAL;
    const int esize = b->dtype == AT_GRPO_BF16 ? 2 : 4;
    if ((static_cast<int64_t>(b->H) * esize) % 128 != 0) return AT_GRPO_EUNSUPPORTED;
  }
  return AT_GRPO_OK;
}

int check_pointers(const at_grpo_batch* b, bool need_tensors) {
  if (!b->cu_seqlens) return AT_GRPO_EINVAL;
  if (b->n_heads > 1 && (!b->resp_agent || !b->head_of_agent || b->n_agent <= 0)) return AT_GRPO_EINVAL;
  if (need_tensors) {
    if (!b->hidden || !b->W || !b->token_id) return AT_GRPO_EINVAL;
    if (reinterpret_cast<uintptr_t>(b->hidden) & 15) return AT_GRPO_EINVAL;
    for (int m = 0; m < b->n_heads; ++m)
      if (!b->W[m] || (reinterpret_cast<uintptr_t>(b->W[m]) & 15)) return AT_GRPO_EINVAL;
  }
  return AT_GRPO_OK;
}

// Lays the workspace out.  Only sizes are read from the batch.
void make_plan(const at_grpo_batch* b, int call, WsAlloc& ws, Plan* p) {
  const int64_t n_tok = b->n_tok;
  const int M = b->n_heads;
  p->L.n_tok = n_tok;
  p->L.n_resp = b->n_resp;
  p->L.n_heads = M;
  p->L.n_agent = b->n_agent;
  p->L.V = b->V;
  p->L.cu_seqlens = b->cu_seqlens;
  p->L.token_id = b->token_id;
  p->L.mask = b->mask;
  p->L.resp_agent = b->resp_agent;
  p->L.head_of_agent = b->head_of_agent;

  TokenScratch& S = p->S;
  S.n_blk = ceil_div(n_tok, kTokPerBlock);
  S.n_blk256 = ceil_div(n_tok, 256);
  S.err = ws.take<int32_t>(64);
  S.cnt = ws.take<int32_t>(kMaxHeads);
  S.resp_cnt = ws.take<int32_t>(kMaxHeads);
  S.resp_of_tok = ws.take<int32_t>(static_cast<size_t>(n_tok));
  S.flag = ws.take<int32_t>(static_cast<size_t>(n_tok));
  S.blk_cnt = ws.take<int32_t>(static_cast<size_t>(M * S.n_blk));
  S.blk_off = ws.take<int32_t>(static_cast<size_t>(M * S.n_blk));
  S.resp_len = ws.take<int32_t>(static_cast<size_t>(b->n_resp));
  S.resp_sum = ws.take<float>(static_cast<size_t>(b->n_resp));
  S.resp_head = ws.take<int32_t>(static_cast<size_t>(b->n_resp));
  const bool heads = call != AT_GRPO_CALL_SURROGATE;
  S.idx = heads ? ws.take<int32_t>(static_cast<size_t>(M) * static_cast<size_t>(n_tok)) : nullptr;
  if (!heads) return;

  HeadGeom& g = p->g;
  g.dtype = b->dtype;
  g.H = b->H;
  g.V = b->V;
  g.esize = b->dtype == AT_GRPO_BF16 ? 2 : 4;
  g.Vp = static_cast<int>(round_up(static_cast<size_t>(b->V), 64));
  g.n_vtiles = static_cast<int>(ceil_div(b->V, 256));
  int64_t tc = static_cast<int64_t>(round_up(static_cast<size_t>(n_tok), 256));
  const bool step = call == AT_GRPO_CALL_POLICY_LOSS_FWD_BWD;
  const bool bwd = call == AT_GRPO_CALL_POLICY_LOSS_BWD || step;
  const int64_t tc_max = bwd ? kMaxChunkTokens : kSubChunkTokens;
  if (tc > tc_max) tc = tc_max;
  if (bwd) {
    int64_t cap = static_cast<int64_t>(kDzBudgetBytes / (static_cast<size_t>(g.Vp) * g.esize)) / 256 * 256;
    if (cap < 256) cap = 256;
    if (tc > cap) tc = cap;
  }
  g.TC = static_cast<int>(tc);
  p->n_chunks = static_cast<int>(ceil_div(n_tok, tc));
  // bf16 backward: two launches of dZ / dHidden per full super-chunk (the fp32 path keeps a transposed
  // copy of dZ whose row stride is the chunk length, and is launched once per chunk)
  int64_t sub_rows = static_cast<int64_t>(kSubChunkBytes / (static_cast<size_t>(g.H) * g.esize)) / 256 * 256;
  if (sub_rows > kSubChunkTokens) sub_rows = kSubChunkTokens;
  while (sub_rows > 256 && kMaxChunkTokens % sub_rows != 0) sub_rows -= 256;
  p->sub = (bwd && g.dtype == AT_GRPO_BF16 && tc == kMaxChunkTokens && sub_rows >= 2048) ? static_cast<int>(sub_rows)
                                                                                           : g.TC;

  if (call == AT_GRPO_CALL_TOKEN_LOGPROB || call == AT_GRPO_CALL_POLICY_LOSS_FWD ||
      call == AT_GRPO_CALL_TOKEN_ENTROPY) {
    const size_t np = static_cast<size_t>(g.n_vtiles) * static_cast<size_t>(g.TC);
    p->part_m = ws.take<float>(np);
    p->part_s = ws.take<float>(np);
    p->part_u = call == AT_GRPO_CALL_TOKEN_ENTROPY ? ws.take<float>(np) : nullptr;
    p->zy = ws.take<float>(static_cast<size_t>(g.TC));
  }
  if (step) {
    // a second compaction (flags, counts, lists) beside the one of S, whose list serves the other class
    p->SB = S;
    p->SF = S;
    p->SB.flag = ws.take<int32_t>(static_cast<size_t>(n_tok));
    p->SF.flag = ws.take<int32_t>(static_cast<size_t>(n_tok));
    p->SB.cnt = ws.take<int32_t>(kMaxHeads);
    p->SF.cnt = ws.take<int32_t>(kMaxHeads);
    p->SF.idx = ws.take<int32_t>(static_cast<size_t>(M) * static_cast<size_t>(n_tok));
    p->gF = g;
    p->gF.TC = static_cast<int>(tc < kSubChunkTokens ? tc : kSubChunkTokens);
    const size_t rows = static_cast<size_t>(p->sub > p->gF.TC ? p->sub : p->gF.TC);   // rows of the largest launch
    const size_t np = static_cast<size_t>(g.n_vtiles) * rows;
    p->part_m = ws.take<float>(np);
    p->part_s = ws.take<float>(np);
    p->part_u = nullptr;
    p->zy = ws.take<float>(rows);
    p->c2 = ws.take<float>(rows);
    p->scale = ws.take<float>(static_cast<size_t>(g.TC));
    p->n_gates = M * p->n_chunks * (g.TC / p->sub);
    p->gates = ws.take<int32_t>(static_cast<size_t>(p->n_gates));
    p->perm = ws.take<int32_t>(static_cast<size_t>(g.TC));
    p->holes = ws.take<int32_t>(static_cast<size_t>(g.TC));
    p->movers = ws.take<int32_t>(static_cast<size_t>(g.TC));
    p->live_cnt = ws.take<int32_t>(64);
  }
  if (bwd) {
    p->coef = step ? nullptr : ws.take<float>(static_cast<size_t>(n_tok));
    p->Wt = ws.take<char>(static_cast<size_t>(g.H) * g.Vp * g.esize);
    p->hT = ws.take<char>(static_cast<size_t>(g.H) * g.TC * g.esize);
    p->dZ = ws.take<char>(static_cast<size_t>(g.TC) * g.Vp * g.esize);
    p->dZt = (g.dtype == AT_GRPO_F32) ? ws.take<char>(static_cast<size_t>(g.V) * g.TC * g.esize) : nullptr;
  }
}

int check_workspace(void* workspace, size_t have, size_t need) {
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || have < need) return AT_GRPO_EWORKSPACE;
  return AT_GRPO_OK;
}

// log-probabilities of the rows on the per-head lists of S, in launches of g.TC rows
int enqueue_logprob_lists(const at_grpo_batch* b, const Plan& p, const HeadGeom& g, const TokenScratch& S,
                          float* logp, float* lse, float* entropy, hipStream_t s) {
  float* part_u = entropy ? p.part_u : nullptr;
  const int n_chunks = static_cast<int>(ceil_div(p.L.n_tok, g.TC));
  for (int m = 0; m < b->n_heads; ++m) {
    for (int c = 0; c < n_chunks; ++c) {
      const HeadChunk ch{S.idx + static_cast<size_t>(m) * p.L.n_tok, S.cnt + m, c * g.TC};
      ATG_TRY(launch_head_fwd(g, ch, b->hidden, b->W[m], b->token_id, p.part_m, p.part_s, part_u, p.zy, s));
      ATG_TRY(launch_lse_combine(g, ch, p.part_m, p.part_s, part_u, p.zy, logp, lse, entropy, s));
    }
  }
  return AT_GRPO_OK;
}

int enqueue_logprob(const at_grpo_batch* b, const Plan& p, float* logp, float* lse, float* entropy,
                    hipStream_t s) {
  ATG_TRY(launch_route(p.L, p.S, s));
  ATG_TRY(launch_compact(p.L, p.S, true, s));
  ATG_TRY(launch_zero_nonparticipating(p.L, p.S, logp, lse, s));
  if (entropy) ATG_TRY(launch_zero_nonparticipating(p.L, p.S, entropy, nullptr, s));
  return enqueue_logprob_lists(b, p, p.g, p.S, logp, lse, entropy, s);
}

bool agg_ok(int agg) { return agg == AT_GRPO_AGG_TOKEN_MEAN || agg == AT_GRPO_AGG_SEQ_MEAN_TOKEN_MEAN; }
bool eps_ok(float lo, float hi) { return lo >= 0.f && lo < 1.f && hi >= 0.f; }

}  // namespace
}  // namespace atg

using namespace atg;

extern "C" size_t at_grpo_workspace_bytes(int32_t which_call, const at_grpo_batch* batch, int32_t n_resp,
                                          int32_t n_env, int32_t n_agent, int32_t n_turn) {
  if (which_call == AT_GRPO_CALL_GROUP_ADVANTAGE)
    return group_advantage_workspace(n_resp, n_env, n_agent, n_turn);
  if (which_call == AT_GRPO_CALL_HEAD_UPDATE) return head_update_workspace();
  if (which_call == AT_GRPO_CALL_DIAGNOSTICS) {
    if (check_layout(batch, false) != AT_GRPO_OK) return 0;
    return diagnostics_workspace(batch->n_resp);
  }
  if ((which_call < AT_GRPO_CALL_TOKEN_LOGPROB || which_call > AT_GRPO_CALL_SURROGATE) &&
      which_call != AT_GRPO_CALL_TOKEN_ENTROPY && which_call != AT_GRPO_CALL_POLICY_LOSS_FWD_BWD)
    return 0;
  if (which_call == AT_GRPO_CALL_POLICY_LOSS_FWD_BWD && batch && batch->dtype == AT_GRPO_F32) {
    // fp32 runs the two calls one after the other in the same workspace
    const size_t f = at_grpo_workspace_bytes(AT_GRPO_CALL_POLICY_LOSS_FWD, batch, n_resp, n_env, n_agent, n_turn);
    const size_t w = at_grpo_workspace_bytes(AT_GRPO_CALL_POLICY_LOSS_BWD, batch, n_resp, n_env, n_agent, n_turn);
    return f > w ? f : w;
  }
  const bool tensors = which_call != AT_GRPO_CALL_SURROGATE;
  if (check_layout(batch, tensors) != AT_GRPO_OK) return 0;
  WsAlloc ws(nullptr);
  Plan p{};
  make_plan(batch, which_call, ws, &p);
  return ws.bytes();
}

extern "C" int at_grpo_token_logprob(const at_grpo_batch* batch, float* logp, float* lse, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
  ATG_TRY(check_layout(batch, true));
  ATG_TRY(check_pointers(batch, true));
  if (!logp) return AT_GRPO_EINVAL;
  WsAlloc ws(workspace);
  Plan p{};
  make_plan(batch, AT_GRPO_CALL_TOKEN_LOGPROB, ws, &p);
  ATG_TRY(check_workspace(workspace, workspace_bytes, ws.bytes()));
  return enqueue_logprob(batch, p, logp, lse, nullptr, static_cast<hipStream_t>(hip_stream));
}

extern "C" int at_grpo_token_entropy(const at_grpo_batch* batch, float* logp, float* lse, float* entropy,
                                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  ATG_TRY(check_layout(batch, true));
  ATG_TRY(check_pointers(batch, true));
  if (!logp || !entropy) return AT_GRPO_EINVAL;
  WsAlloc ws(workspace);
  Plan p{};
  make_plan(batch, AT_GRPO_CALL_TOKEN_ENTROPY, ws, &p);
  ATG_TRY(check_workspace(workspace, workspace_bytes, ws.bytes()));
  return enqueue_logprob(batch, p, logp, lse, entropy, static_cast<hipStream_t>(hip_stream));
}

extern "C" int at_grpo_surrogate_from_logp(const at_grpo_batch* batch, const float* logp,
                                           const float* old_logp, const float* adv, float eps_low,
                                           float eps_high, int32_t agg, float* loss, uint8_t* clip_mask,
                                           int32_t* n_valid, void* workspace, size_t workspace_bytes,
                                           void* hip_stream) {
  ATG_TRY(check_layout(batch, false));
  ATG_TRY(check_pointers(batch, false));
  if (!logp || !old_logp || !adv || !loss) return AT_GRPO_EINVAL;
  if (!agg_ok(agg) || !eps_ok(eps_low, eps_high)) return AT_GRPO_EINVAL;
  WsAlloc ws(workspace);
  Plan p{};
  make_plan(batch, AT_GRPO_CALL_SURROGATE, ws, &p);
  ATG_TRY(check_workspace(workspace, workspace_bytes, ws.bytes()));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  ATG_TRY(launch_fill_i32(p.S.err, 1, 0, s));
  return launch_surrogate(p.L, p.S, logp, old_logp, adv, eps_low, eps_high, agg, loss, clip_mask, n_valid, s);
}

extern "C" int at_grpo_surrogate_diagnostics(const at_grpo_batch* batch, const float* logp,
                                             const float* old_logp, const float* adv, float eps_low,
                                             float eps_high, int32_t* counts, float* stats, void* workspace,
                                             size_t workspace_bytes, void* hip_stream) {
  ATG_TRY(check_layout(batch, false));
  ATG_TRY(check_pointers(batch, false));
  if (!logp || !old_logp || !adv || !counts || !stats) return AT_GRPO_EINVAL;
  if (!eps_ok(eps_low, eps_high)) return AT_GRPO_EINVAL;
  ATG_TRY(check_workspace(workspace, workspace_bytes, diagnostics_workspace(batch->n_resp)));
  WsAlloc ws(nullptr);
  Plan p{};
  make_plan(batch, AT_GRPO_CALL_SURROGATE, ws, &p);   // layout only; the scratch is laid out by the launcher
  return launch_diagnostics(p.L, logp, old_logp, adv, eps_low, eps_high, counts, stats, workspace,
                            static_cast<hipStream_t>(hip_stream));
}

extern "C" int at_grpo_policy_loss_fwd(const at_grpo_batch* batch, const float* old_logp, const float* adv,
                                       float eps_low, float eps_high, int32_t agg, float* loss, float* logp,
                                       float* lse, uint8_t* clip_mask, int32_t* n_valid, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  ATG_TRY(check_layout(batch, true));
  ATG_TRY(check_pointers(batch, true));
  if (!old_logp || !adv || !loss || !logp || !lse) return AT_GRPO_EINVAL;
  if (!agg_ok(agg) || !eps_ok(eps_low, eps_high)) return AT_GRPO_EINVAL;
  WsAlloc ws(workspace);
  Plan p{};
  make_plan(batch, AT_GRPO_CALL_POLICY_LOSS_FWD, ws, &p);
  ATG_TRY(check_workspace(workspace, workspace_bytes, ws.bytes()));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  ATG_TRY(enqueue_logprob(batch, p, logp, lse, nullptr, s));
  return launch_surrogate(p.L, p.S, logp, old_logp, adv, eps_low, eps_high, agg, loss, clip_mask, n_valid, s);
}

extern "C" int at_grpo_policy_loss_bwd(const at_grpo_batch* batch, const float* old_logp, const float* adv,
                                       const float* logp, const float* lse, float eps_low, float eps_high,
                                       int32_t agg, const float* grad_loss, void* d_hidden,
                                       float* const* dW, int32_t accumulate_dW, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  ATG_TRY(check_layout(batch, true));
  ATG_TRY(check_pointers(batch, true));
  if (!old_logp || !adv || !logp || !lse || !d_hidden || !dW) return AT_GRPO_EINVAL;
  if (reinterpret_cast<uintptr_t>(d_hidden) & 15) return AT_GRPO_EINVAL;
  for (int m = 0; m < batch->n_heads; ++m)
    if (!dW[m]) return AT_GRPO_EINVAL;
  if (!agg_ok(agg) || !eps_ok(eps_low, eps_high)) return AT_GRPO_EINVAL;
  WsAlloc ws(workspace);
  Plan p{};
  make_plan(batch, AT_GRPO_CALL_POLICY_LOSS_BWD, ws, &p);
  ATG_TRY(check_workspace(workspace, workspace_bytes, ws.bytes()));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  // participation and weights, then the coefficient; rows with g_t = 0 drop out of the lists
  ATG_TRY(launch_route(p.L, p.S, s));
  ATG_TRY(launch_compact(p.L, p.S, false, s));
  if (agg == AT_GRPO_AGG_SEQ_MEAN_TOKEN_MEAN) ATG_TRY(launch_resp_len(p.L, p.S, s));
  ATG_TRY(launch_coef(p.L, p.S, logp, old_logp, adv, eps_low, eps_high, agg, grad_loss, p.coef, s));
  ATG_TRY(launch_compact(p.L, p.S, true, s));
  ATG_TRY(launch_fill_bytes16(d_hidden, p.L.n_tok * static_cast<int64_t>(p.g.H) * p.g.esize, s));

  for (int m = 0; m < batch->n_heads; ++m) {
    ATG_TRY(launch_transpose_w(p.g, batch->W[m], p.Wt, s));
    for (int c = 0; c < p.n_chunks; ++c) {
      const HeadChunk ch{p.S.idx + static_cast<size_t>(m) * p.L.n_tok, p.S.cnt + m, c * p.g.TC};
      ATG_TRY(launch_gather_transpose_hidden(p.g, ch, batch->hidden, p.hT, s));
      HeadGeom gs = p.g;
      gs.TC = p.sub;
      for (int c1 = 0; c1 < p.g.TC; c1 += p.sub) {
        const HeadChunk sub{ch.idx, ch.cnt, ch.c0 + c1};
        char* dZ_sub = static_cast<char*>(p.dZ) + static_cast<size_t>(c1) * p.g.Vp * p.g.esize;
        ATG_TRY(launch_head_dz(gs, sub, batch->hidden, batch->W[m], batch->token_id, lse, p.coef, dZ_sub,
                               p.dZt, s));
        ATG_TRY(launch_head_dh(gs, sub, dZ_sub, p.Wt, d_hidden, s));
      }
      ATG_TRY(launch_head_dw(p.g, ch, p.dZ, p.dZt, p.hT, dW[m], (accumulate_dW != 0 || c > 0) ? 1 : 0,
                             c == 0 ? 1 : 0, s));
    }
  }
  return AT_GRPO_OK;
}

extern "C" int at_grpo_policy_loss_fwd_bwd(const at_grpo_batch* batch, const float* old_logp, const float* adv,
                                           float eps_low, float eps_high, int32_t agg, const float* grad_loss,
                                           float* loss, float* logp, float* lse, uint8_t* clip_mask,
                                           int32_t* n_valid, void* d_hidden, float* const* dW,
                                           int32_t accumulate_dW, void* workspace, size_t workspace_bytes,
                                           void* hip_stream) {
  ATG_TRY(check_layout(batch, true));
  ATG_TRY(check_pointers(batch, true));
  if (!old_logp || !adv || !loss || !logp || !lse || !d_hidden || !dW) return AT_GRPO_EINVAL;
  if (reinterpret_cast<uintptr_t>(d_hidden) & 15) return AT_GRPO_EINVAL;
  for (int m = 0; m < batch->n_heads; ++m)
    if (!dW[m]) return AT_GRPO_EINVAL;
  if (!agg_ok(agg) || !eps_ok(eps_low, eps_high)) return AT_GRPO_EINVAL;
  if (batch->dtype == AT_GRPO_F32) {
    ATG_TRY(at_grpo_policy_loss_fwd(batch, old_logp, adv, eps_low, eps_high, agg, loss, logp, lse, clip_mask,
                                    n_valid, workspace, workspace_bytes, hip_stream));
    return at_grpo_policy_loss_bwd(batch, old_logp, adv, logp, lse, eps_low, eps_high, agg, grad_loss, d_hidden,
                                   dW, accumulate_dW, workspace, workspace_bytes, hip_stream);
  }
  WsAlloc ws(workspace);
  Plan p{};
  make_plan(batch, AT_GRPO_CALL_POLICY_LOSS_FWD_BWD, ws, &p);
  ATG_TRY(check_workspace(workspace, workspace_bytes, ws.bytes()));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  // participation; the weights of Eq. (2) count every participating row, whatever its advantage
  ATG_TRY(launch_route(p.L, p.S, s));
  ATG_TRY(launch_compact(p.L, p.S, false, s));
  if (agg == AT_GRPO_AGG_SEQ_MEAN_TOKEN_MEAN) ATG_TRY(launch_resp_len(p.L, p.S, s));
  ATG_TRY(launch_zero_nonparticipating(p.L, p.S, logp, lse, s));
  // rows of responses with a zero advantage carry no gradient: they only need their log-probability
  ATG_TRY(launch_split_by_advantage(p.L, p.S, adv, p.SB.flag, p.SF.flag, s));
  ATG_TRY(launch_compact(p.L, p.SF, true, s));
  ATG_TRY(launch_compact(p.L, p.SB, true, s));
  ATG_TRY(enqueue_logprob_lists(batch, p, p.gF, p.SF, logp, lse, nullptr, s));
  ATG_TRY(launch_fill_bytes16(d_hidden, p.L.n_tok * static_cast<int64_t>(p.g.H) * p.g.esize, s));
  ATG_TRY(launch_fill_i32(p.gates, p.n_gates, 0, s));
  const CoefArgs ca = make_coef_args(p.S, old_logp, adv, eps_low, eps_high, agg, grad_loss);

  int gate_no = 0;
  for (int m = 0; m < batch->n_heads; ++m) {
    ATG_TRY(launch_transpose_w(p.g, batch->W[m], p.Wt, s));
    for (int c = 0; c < p.n_chunks; ++c) {
      const HeadChunk ch{p.SB.idx + static_cast<size_t>(m) * p.L.n_tok, p.SB.cnt + m, c * p.g.TC};
      HeadGeom gs = p.g;
      gs.TC = p.sub;
      for (int c1 = 0; c1 < p.g.TC; c1 += p.sub) {
        const HeadChunk sub{ch.idx, ch.cnt, ch.c0 + c1};
        char* E_sub = static_cast<char*>(p.dZ) + static_cast<size_t>(c1) * p.g.Vp * p.g.esize;
        float* scale_sub = p.scale + c1;
        int32_t* gate = p.gates + gate_no++;
        ATG_TRY(launch_ref_logit(gs, sub, batch->hidden, batch->W[m], batch->token_id, p.c2, s));
        ATG_TRY(launch_head_fe(gs, sub, batch->hidden, batch->W[m], batch->token_id, p.c2, E_sub, p.part_s, p.zy, s));
        ATG_TRY(launch_fe_combine(gs, sub, m, p.part_s, p.c2, p.zy, batch->token_id, ca, logp, lse, scale_sub,
                                  E_sub, gate, s));
        // exponent range exceeded somewhere in this launch: the two-pass kernels redo it (they return at once
        // otherwise)
        ATG_TRY(launch_head_fwd(gs, sub, batch->hidden, batch->W[m], batch->token_id, p.part_m, p.part_s, nullptr,
                                p.zy, s, gate));
        ATG_TRY(launch_lse_combine(gs, sub, p.part_m, p.part_s, nullptr, p.zy, logp, lse, nullptr, s, gate));
        ATG_TRY(launch_fallback_scale(gs, sub, m, ca, logp, scale_sub, gate, s));
        ATG_TRY(launch_head_dz(gs, sub, batch->hidden, batch->W[m], batch->token_id, lse, nullptr, E_sub, nullptr, s,
                               gate));
      }
      // rows on the clipped branch (factor 0) are taken out of the chunk before the two contractions
      // (d_hidden is zero there already); one dHidden launch over the whole super-chunk, so that the rows left
      // fill the grid evenly
      ATG_TRY(launch_compact_rows(p.g, ch, p.scale, p.dZ, p.perm, p.holes, p.movers, p.live_cnt, p.live_cnt + 1, s));
      ATG_TRY(launch_head_dh(p.g, ch, p.dZ, p.Wt, d_hidden, s, p.scale, p.perm, p.live_cnt));
      ATG_TRY(launch_gather_transpose_hidden(p.g, ch, batch->hidden, p.hT, s, p.scale, p.perm, p.live_cnt));
      ATG_TRY(launch_head_dw(p.g, ch, p.dZ, nullptr, p.hT, dW[m], (accumulate_dW != 0 || c > 0) ? 1 : 0,
                             c == 0 ? 1 : 0, s, p.live_cnt));
    }
  }
  return launch_surrogate(p.L, p.S, logp, old_logp, adv, eps_low, eps_high, agg, loss, clip_mask, n_valid, s);
}

extern "C" const char* at_grpo_status_string(int32_t status) {
  switch (status) {
    case AT_GRPO_OK: return "ok";
    case AT_GRPO_EINVAL: return "invalid argument";
    case AT_GRPO_EUNSUPPORTED: return "unsupported dtype or shape";
    case AT_GRPO_EWORKSPACE: return "workspace missing, misaligned or too small";
    case AT_GRPO_EHIP: return "HIP runtime error";
    case AT_GRPO_ESCRATCH: return "input exceeds the library's fixed scratch array (use the call that takes a workspace)";
    default: return "unknown status";
  }
}

extern "C" int32_t at_grpo_version(void) { return 100; }

extern "C" int at_grpo_profile_enable(int32_t on) {
  for (int c = 0; c < PROF_N; ++c) {
    for (auto& e : g_prof.ev[c]) {
      (void)hipEventDestroy(e.first);
      (void)hipEventDestroy(e.second);
    }
    g_prof.ev[c].clear();
  }
  g_prof.on = on != 0;
  return AT_GRPO_OK;
}

extern "C" int32_t at_grpo_profile_classes(void) { return PROF_N; }

extern "C" int at_grpo_profile_read(int32_t which, const char** name, int64_t* launches, double* total_ms) {
  if (which < 0 || which >= PROF_N || !launches || !total_ms) return AT_GRPO_EINVAL;
  if (name) *name = kProfNames[which];
  double tot = 0.0;
  int64_t n = 0;
  for (auto& e : g_prof.ev[which]) {
    ATG_HIP_TRY(hipEventSynchronize(e.second));
    float ms = 0.f;
    ATG_HIP_TRY(hipEventElapsedTime(&ms, e.first, e.second));
    tot += ms;
    ++n;
  }
  *launches = n;
  *total_ms = tot;
  return AT_GRPO_OK;
}
