/*
 * at_grpo.h -- C ABI of the MI355X (gfx950) AT-GRPO policy-loss library.
 *
 * The library computes, on one GPU, the per-token policy loss of AT-GRPO
 * (arXiv 2510.11062): agent- and turn-wise grouped advantages (Alg. 1, Phase 1; Eq. 1),
 * log pi_theta(token) from the LM head (the ratio below Eq. 2), the clipped surrogate with
 * masked averaging per policy (Eq. 2; per-model batches B_m of Sec. 3) and its gradients
 * with respect to the final hidden states and the head weights.
 *
 * Conventions common to every call
 *   - Pointers are DEVICE pointers unless the comment says "host".  The caller owns every
 *     buffer; the library never allocates, frees or keeps a pointer after the call returns.
 *   - All work is enqueued on `hip_stream` (a hipStream_t cast to void*; NULL = default
 *     stream).  No call synchronises with the host.  Scalar results live in device memory.
 *   - `workspace` is caller-provided device scratch of at least at_grpo_workspace_bytes()
 *     bytes, 256-byte aligned.  Its first int32 is an error word: 0, or the bit-or of
 *     AT_GRPO_DATA_* flags raised by data that is only visible on the device.  Offending
 *     elements are treated as masked out.  Read it after synchronising the stream.
 *   - Return value: an at_grpo_status.  Argument errors are detected on the host before
 *     anything is launched; nothing is thrown and nothing aborts.
 *   - Matrices are row-major and dense.  `hidden` is [n_tok, H]; each head W is [V, H].
 *   - dtype AT_GRPO_BF16 requires H % 64 == 0; AT_GRPO_F32 requires H % 32 == 0.
 */
#ifndef AT_GRPO_H_
#define AT_GRPO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AT_GRPO_OK = 0,
  AT_GRPO_EINVAL = 1,       /* null pointer, non-positive size, inconsistent arguments */
  AT_GRPO_EUNSUPPORTED = 2, /* dtype / shape the kernels do not cover                 */
  AT_GRPO_EWORKSPACE = 3,   /* workspace missing, misaligned or too small             */
  AT_GRPO_EHIP = 4,         /* a HIP runtime call or kernel launch failed             */
  AT_GRPO_ESCRATCH = 5      /* input too large for the library's fixed scratch array  */
} at_grpo_status;

typedef enum { AT_GRPO_F32 = 0, AT_GRPO_BF16 = 1 } at_grpo_dtype;

/* How Eq. (2)'s expectation over the per-model batch is taken (the paper writes a mean over
 * groups and candidates; credit is per response token, Sec. 4.1):
 *   TOKEN_MEAN           loss_m = -(1/n_m) sum_t l_t          over the n_m response tokens of B_m
 *   SEQ_MEAN_TOKEN_MEAN  loss_m = -(1/R_m) sum_r (1/len_r) sum_{t in r} l_t                  */
typedef enum { AT_GRPO_AGG_TOKEN_MEAN = 0, AT_GRPO_AGG_SEQ_MEAN_TOKEN_MEAN = 1 } at_grpo_agg;

/* F_norm of Eq. (1): the group's standard deviation (plus eps_std), or 1. */
typedef enum { AT_GRPO_NORM_STD = 0, AT_GRPO_NORM_NONE = 1 } at_grpo_norm;

/* Which responses form a group in Eq. (1): the paper's agent- and turn-wise key, or one of the two
 * groupings it argues against (Sec. 4.1, Fig. 3; Sec. 5.3), kept for comparison runs. */
typedef enum {
  AT_GRPO_GROUP_BY_AGENT_TURN = 0, /* (e, i, t): AT-GRPO, Alg. 1                                      */
  AT_GRPO_GROUP_BY_TRAJECTORY = 1, /* e alone: every candidate of a task in one group (GRPO on the MAS) */
  AT_GRPO_GROUP_BY_PARALLEL = 2    /* (e, i, t) at t = 0, one group per candidate at t > 0: what
                                      sampling K whole trajectories in parallel yields               */
} at_grpo_group_by;

/* Bits of the device error word (workspace[0]). */
enum {
  AT_GRPO_DATA_ID_RANGE = 1,     /* env/agent/turn id outside its extent              */
  AT_GRPO_DATA_REWARD = 2,       /* non-finite reward (the response then takes no part) */
  AT_GRPO_DATA_TOKEN_RANGE = 4,  /* token_id outside [0, V) on an unmasked row        */
  AT_GRPO_DATA_SEQLENS = 8,      /* cu_seqlens not monotone within [0, n_tok]         */
  AT_GRPO_DATA_AGENT_RANGE = 16  /* resp_agent / head_of_agent entry out of range     */
};

/* Bits of clip_mask[t] (Eq. 2's clip, decided in log space on d = logp - old_logp, one fp32
 * subtraction, against lo = (float)log1p(-eps_low) and hi = (float)log1p(eps_high)). */
enum {
  AT_GRPO_CLIP_LOW = 1,       /* d < lo : ratio below 1 - eps_low                    */
  AT_GRPO_CLIP_HIGH = 2,      /* d > hi : ratio above 1 + eps_high                   */
  AT_GRPO_CLIP_ZERO_GRAD = 4  /* min() selects the clipped branch: no gradient       */
};

/* Which call a workspace is sized for. */
typedef enum {
  AT_GRPO_CALL_GROUP_ADVANTAGE = 0,
  AT_GRPO_CALL_TOKEN_LOGPROB = 1,
  AT_GRPO_CALL_POLICY_LOSS_FWD = 2,
  AT_GRPO_CALL_POLICY_LOSS_BWD = 3,
  AT_GRPO_CALL_SURROGATE = 4,
  AT_GRPO_CALL_HEAD_UPDATE = 5,  /* size does not depend on the other arguments */
  AT_GRPO_CALL_DIAGNOSTICS = 6,
  AT_GRPO_CALL_TOKEN_ENTROPY = 7,
  AT_GRPO_CALL_POLICY_LOSS_FWD_BWD = 8
} at_grpo_call;

/*
 * A batch of rollout tokens (Alg. 1 Phase 2: the per-model batches B_m, all models at once).
 * Row t of `hidden` is the final hidden state that predicts token_id[t].  Response r owns rows
 * [cu_seqlens[r], cu_seqlens[r+1]); rows owned by no response, and rows with mask 0, take no
 * part (packed layout: mask == NULL; padded layout: fixed-size slots plus mask).  With
 * n_heads > 1 the rows of response r go to head head_of_agent[resp_agent[r]] (the role
 * mapping sigma of Sec. 3); with n_heads == 1 both arrays may be NULL.
 */
typedef struct {
  int32_t dtype;             /* at_grpo_dtype of hidden and W                            */
  int32_t H, V, n_heads;     /* n_heads in [1, 16]                                       */
  int64_t n_tok;             /* rows of hidden / token_id / mask (padding included)      */
  int32_t n_resp;            /* R                                                        */
  int32_t n_agent;           /* length of head_of_agent (ignored if n_heads == 1)        */
  const int64_t* cu_seqlens; /* [R+1] device                                             */
  const void* hidden;        /* [n_tok, H] device                                        */
  const void* const* W;      /* HOST array of n_heads device pointers, each [V, H]       */
  const int32_t* token_id;   /* [n_tok] device, sampled token, 0 <= id < V               */
  const uint8_t* mask;       /* [n_tok] device or NULL (all ones)                        */
  const int32_t* resp_agent; /* [R] device or NULL                                       */
  const int32_t* head_of_agent; /* [n_agent] device or NULL                              */
} at_grpo_batch;

/*
 * Agent- and turn-wise grouping and group-relative advantages.
 * Alg. 1 ("Define group key g <- hash(e, i, t) and compute advantages"), Sec. 4.1
 * "Agent- and Turn-wise Grouping", Eq. (1).
 *
 * key(r) = (env_id[r] * n_agent + agent_id[r]) * n_turn + turn_id[r]; groups are numbered
 * densely in ascending key order; keys that do not occur produce no group.
 *   group_id[R]      dense group of each response (-1 for a response with an id out of range or a
 *                    non-finite reward: it joins no group, gets advantage 0 and does not touch the
 *                    statistics of the others)
 *   n_groups[1]      G
 *   seg_offsets[G+1] CSR offsets into perm; the buffer must hold min(R, n_env*n_agent*n_turn)+1
 *   perm[R]          responses sorted by key, ties in ascending original index (stable)
 *   adv[R]           (reward - mean_g) / (std_g + eps_std)   [NORM_STD]   or reward - mean_g
 *                    [NORM_NONE]; std uses divisor n_g - ddof (0 if that is <= 0); a group
 *                    whose rewards are all the same fp32 value gets exactly 0
 *   group_mean[G], group_std[G]  optional (NULL to skip)
 * ddof is 0 or 1.  Arithmetic is fp32, two passes (mean, then squared deviations): groups of up to 16
 * members are summed sequentially in perm order, larger ones as 64 lane-strided partial sums (member
 * j of the group goes to partial j mod 64) that are combined in a fixed order; either way the result
 * does not depend on the order in which the responses arrive or on the run.
 */
int at_grpo_group_advantage(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn,
                            const int32_t* env_id, const int32_t* agent_id, const int32_t* turn_id,
                            const float* reward, float eps_std, int32_t ddof, int32_t norm,
                            int32_t* group_id, int32_t* n_groups, int32_t* seg_offsets,
                            int32_t* perm, float* adv, float* group_mean, float* group_std,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * at_grpo_group_advantage under another grouping key (`group_by`, see at_grpo_group_by): everything
 * else, including the canonical numbering (ascending key), is the same.
 *   TRAJECTORY  key = e: agent_id and turn_id are only range-checked; seg_offsets needs min(R, n_env) + 1
 *   PARALLEL    key = ((e * n_agent + i) * n_turn + t) * n_sample + (t > 0 ? sample_id[r] : 0), with
 *               sample_id[R] the candidate index c in [0, n_sample): every group at t > 0 is a single
 *               response and gets advantage 0 (the degenerate case Sec. 4.1 describes);
 *               seg_offsets needs min(R, n_env * n_agent * n_turn * n_sample) + 1 entries
 * sample_id and n_sample are ignored otherwise.  Workspace: at_grpo_group_advantage_keyed_workspace_bytes.
 */
int at_grpo_group_advantage_keyed(int32_t group_by, int32_t n_resp, int32_t n_env, int32_t n_agent,
                                  int32_t n_turn, int32_t n_sample, const int32_t* env_id,
                                  const int32_t* agent_id, const int32_t* turn_id, const int32_t* sample_id,
                                  const float* reward, float eps_std, int32_t ddof, int32_t norm,
                                  int32_t* group_id, int32_t* n_groups, int32_t* seg_offsets, int32_t* perm,
                                  float* adv, float* group_mean, float* group_std, void* workspace,
                                  size_t workspace_bytes, void* hip_stream);
size_t at_grpo_group_advantage_keyed_workspace_bytes(int32_t group_by, int32_t n_resp, int32_t n_env,
                                                     int32_t n_agent, int32_t n_turn, int32_t n_sample);

/*
 * The same with the step in front of it: agent-wise credit assignment, Eq. (3) of Sec. 4.1,
 *   reward[r] = alpha * r_team[r] + r_loc[r]     (one fp32 multiplication, then one fp32 addition)
 * feeds Eq. (1), and the greedy choice of tree-structured sampling (Alg. 1, "c* <- arg max_c r^(c)")
 * is taken on the same groups:
 *   reward[R]   output, the mixed reward (also what adv, group_mean, group_std are computed from)
 *   best[G]     optional (NULL to skip): response index of the candidate with the largest reward of
 *               each group, the lowest response index among equal rewards; the buffer must hold
 *               min(R, n_env*n_agent*n_turn) entries
 * r_team[R], r_loc[R] are inputs; alpha must be finite.  Every other argument, the workspace size
 * (AT_GRPO_CALL_GROUP_ADVANTAGE) and the error behaviour are those of at_grpo_group_advantage; a
 * non-finite mixed reward raises AT_GRPO_DATA_REWARD.
 */
int at_grpo_group_advantage_mixed(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn,
                                  const int32_t* env_id, const int32_t* agent_id, const int32_t* turn_id,
                                  const float* r_team, const float* r_loc, float alpha, float eps_std,
                                  int32_t ddof, int32_t norm, float* reward, int32_t* group_id,
                                  int32_t* n_groups, int32_t* seg_offsets, int32_t* perm, float* adv,
                                  float* group_mean, float* group_std, int32_t* best, void* workspace,
                                  size_t workspace_bytes, void* hip_stream);

/*
 * at_grpo_group_advantage for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the scratch
 * is a fixed array of at_grpo_static_scratch_bytes() bytes (2 MiB) in the library's own device
 * memory, which every GPU the library runs on holds until the process ends.  The call allocates and
 * frees nothing.  Same inputs, outputs, arithmetic and results as at_grpo_group_advantage, plus
 *   data_error[1]  optional device output (NULL to skip): the error word of this call (AT_GRPO_DATA_*)
 * Limit: at_grpo_workspace_bytes(AT_GRPO_CALL_GROUP_ADVANTAGE, ...) of the same extents must not
 * exceed at_grpo_static_scratch_bytes(), i.e. about 12 * n_resp + 8 * n_env * n_agent * n_turn bytes
 * <= 2 MiB (65 536 responses over 65 536 keys fit, as does every workload of the paper's shape); beyond it the call
 * returns AT_GRPO_ESCRATCH and launches nothing.
 * All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different streams
 * or threads) race and must be serialised by the caller.  Everything the kernels need cleared is
 * cleared by the call itself with fill kernels (no memset nodes), so it may be captured in a graph;
 * the first call on a device looks the array's address up and should be made outside a capture.
 */
size_t at_grpo_static_scratch_bytes(void);
int at_grpo_group_advantage_static(int32_t n_resp, int32_t n_env, int32_t n_agent, int32_t n_turn,
                                   const int32_t* env_id, const int32_t* agent_id, const int32_t* turn_id,
                                   const float* reward, float eps_std, int32_t ddof, int32_t norm,
                                   int32_t* group_id, int32_t* n_groups, int32_t* seg_offsets,
                                   int32_t* perm, float* adv, float* group_mean, float* group_std,
                                   int32_t* data_error, void* hip_stream);

/*
 * log pi_theta(token_id[t]) and the log-sum-exp of the head logits for every participating row
 * (the policy probability inside r(theta) below Eq. 2).  Logits z[t, v] = <hidden[t], W_m[v]>
 * are produced tile by tile on the matrix cores and reduced on the fly; they are never written
 * to memory.  Rows that take no part get logp = lse = 0.
 *   logp[n_tok], lse[n_tok] (lse may be NULL)
 */
int at_grpo_token_logprob(const at_grpo_batch* batch, float* logp, float* lse,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Clipped surrogate of Eq. (2) given log-probs (the stage after the head):
 *   d_t = logp_t - old_logp_t,  r_t = exp(d_t),  A_t = adv[response of t]
 *   l_t = min(r_t A_t, clip(r_t, 1 - eps_low, 1 + eps_high) A_t)
 *   loss[m] = - sum_{t in B_m} w_t l_t      (w_t per `agg`)
 *   clip_mask[n_tok], n_valid[n_heads] (participating rows per head)
 * Only the batch's layout fields are used (n_tok, n_resp, cu_seqlens, mask, token_id for the
 * range check, resp_agent, head_of_agent, n_heads, V); hidden and W may be NULL.
 * The reduction is a fixed-order tree: results are bit-reproducible.
 */
int at_grpo_surrogate_from_logp(const at_grpo_batch* batch, const float* logp, const float* old_logp,
                                const float* adv, float eps_low, float eps_high, int32_t agg,
                                float* loss, uint8_t* clip_mask, int32_t* n_valid,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * at_grpo_token_logprob plus a monitor: the entropy of the next-token distribution at every
 * participating row, H_t = - sum_v p_v ln p_v = lse_t - sum_v p_v z_v, from one more partial sum per
 * vocabulary tile in the same pass (the paper trains with entropy coefficient 0, App. C.1; nothing in
 * the loss uses it).  Rows that take no part get 0.
 *   logp[n_tok], lse[n_tok] (may be NULL), entropy[n_tok]
 * Workspace: AT_GRPO_CALL_TOKEN_ENTROPY.
 */
int at_grpo_token_entropy(const at_grpo_batch* batch, float* logp, float* lse, float* entropy,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Monitors of the clipped-ratio update of Eq. (2), per policy, over the same participating rows as
 * at_grpo_surrogate_from_logp (the paper reports none of them; its entropy coefficient is 0 and Eq. 2
 * carries no KL term):
 *   counts[n_heads][4]  rows, rows with d < lo, rows with d > hi, rows on the clipped branch
 *                       (AT_GRPO_CLIP_LOW / _HIGH / _ZERO_GRAD counted), d = logp - old_logp in fp32
 *   stats[n_heads][2]   mean of exp(d) - 1 - d (sample estimate of KL(pi_old || pi_theta)), mean exp(d)
 * Sums are taken in a fixed order.  Workspace: AT_GRPO_CALL_DIAGNOSTICS (needs batch->n_resp only).
 */
int at_grpo_surrogate_diagnostics(const at_grpo_batch* batch, const float* logp, const float* old_logp,
                                  const float* adv, float eps_low, float eps_high, int32_t* counts,
                                  float* stats, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Forward of the policy loss: at_grpo_token_logprob followed by at_grpo_surrogate_from_logp.
 * Outputs logp[n_tok], lse[n_tok] (both are needed by the backward), loss[n_heads],
 * clip_mask[n_tok], n_valid[n_heads].
 */
int at_grpo_policy_loss_fwd(const at_grpo_batch* batch, const float* old_logp, const float* adv,
                            float eps_low, float eps_high, int32_t agg,
                            float* loss, float* logp, float* lse, uint8_t* clip_mask, int32_t* n_valid,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward of sum_m grad_loss[m] * loss[m] (grad_loss == NULL means all ones):
 *   g_t = -w_t A_t r_t [unclipped branch selected] grad_loss[m]
 *   dZ[t, v]     = g_t (1[v = token_id[t]] - exp(z[t, v] - lse_t))     (logits recomputed)
 *   d_hidden[t]  = sum_v dZ[t, v] W_m[v]          dtype of hidden, [n_tok, H]; rows that take
 *                                                  no part or have g_t = 0 are exactly 0
 *   dW[m][v]     = sum_t dZ[t, v] hidden[t]       fp32 [V, H] per head; dW is a HOST array of
 *                                                  n_heads device pointers; overwritten, or
 *                                                  added to when accumulate_dW != 0
 * logp and lse are the forward's outputs.  Rows with g_t = 0 are skipped entirely.
 */
int at_grpo_policy_loss_bwd(const at_grpo_batch* batch, const float* old_logp, const float* adv,
                            const float* logp, const float* lse,
                            float eps_low, float eps_high, int32_t agg, const float* grad_loss,
                            void* d_hidden, float* const* dW, int32_t accumulate_dW,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * One training step's worth of Eq. (2): at_grpo_policy_loss_fwd followed by at_grpo_policy_loss_bwd
 * (same arguments, same outputs, same error behaviour), computed from ONE pass over the logits.  For
 * AT_GRPO_BF16, rows whose response has a non-zero advantage (only they can carry gradient) have their
 * logits produced once: with the reference c_t = z[t, token_id[t]] (one dot product per row) the forward
 * tile writes e[t, v] = exp(z[t, v] - c_t) in bf16, as dZ would be written, and
 *   lse_t = c_t + ln S_t,  S_t = sum_v e[t, v],   dZ[t, v] = a_t (e[t, v] - S_t 1[v = token_id[t]]),
 *   a_t = -g_t / S_t
 * so that d_hidden and dW follow from e by two contractions and a per-row factor, without recomputing the
 * logits.  A launch in which some S_t leaves [1, 2^60) (the sampled token about e^88 times less likely than
 * the mode, or non-finite inputs) is redone by the two-pass kernels, on the device, without host
 * involvement.  Rows of zero-advantage responses only get logp / lse.  AT_GRPO_F32 runs the two calls one
 * after the other.  Results agree with the two-call sequence to rounding (e and the scaled hidden rows are
 * rounded to bf16 where that path rounds dZ).  Workspace: AT_GRPO_CALL_POLICY_LOSS_FWD_BWD.
 */
int at_grpo_policy_loss_fwd_bwd(const at_grpo_batch* batch, const float* old_logp, const float* adv,
                                float eps_low, float eps_high, int32_t agg, const float* grad_loss,
                                float* loss, float* logp, float* lse, uint8_t* clip_mask, int32_t* n_valid,
                                void* d_hidden, float* const* dW, int32_t accumulate_dW,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Hyper-parameters of the head update (App. C.1: Adam, learning rate 1e-6, weight decay 0.01,
 * gradient clipping at 1.0; beta1, beta2 and eps are not stated there: 0.9, 0.999, 1e-8 are the
 * customary values).
 */
typedef struct {
  float lr, beta1, beta2, eps;
  float weight_decay;
  float max_grad_norm; /* 0 disables clipping                                                    */
  int32_t step;        /* 1 for the first update (bias correction 1 - beta^step)                 */
  int32_t decoupled;   /* 1: w <- w (1 - lr wd) before the step; 0: g <- g + wd w (L2 penalty)   */
} at_grpo_adam;

/*
 * "Update policy m" of Alg. 1 (Phase 2) for the head weights, with App. C.1's recipe:
 *   norm  = L2 norm of dW over all n_heads heads together
 *   g     = dW * min(1, max_grad_norm / (norm + 1e-6))
 *   m     <- beta1 m + (1 - beta1) g,   v <- beta2 v + (1 - beta2) g^2
 *   w     <- w - lr wd w - (lr / (1 - beta1^step)) m / (sqrt(v / (1 - beta2^step)) + eps)
 * (decoupled form; the coupled form adds wd w to g instead).  All arithmetic is fp32.
 *   W        HOST array of n_heads device pointers, each [V, H] in `dtype`, updated in place
 *   W_master HOST array of device pointers to the fp32 weights that are stepped, each [V, H];
 *            required for AT_GRPO_BF16 (W then receives their bf16 rounding, nearest-even);
 *            ignored for AT_GRPO_F32 (W itself is stepped)
 *   dW       HOST array of device pointers, fp32 [V, H] (what at_grpo_policy_loss_bwd produced,
 *            possibly accumulated over several mini-batches); read only
 *   m, v     HOST arrays of device pointers, fp32 [V, H], Adam moments, updated in place
 *   opt      host pointer
 *   grad_norm[2]  device output: the norm before clipping, and the factor applied
 * Every device pointer must be 16-byte aligned; H % 4 == 0.  Workspace: AT_GRPO_CALL_HEAD_UPDATE.
 * The norm is reduced in a fixed order, so results are reproducible run to run.
 */
int at_grpo_head_update(int32_t dtype, int32_t H, int32_t V, int32_t n_heads, void* const* W,
                        float* const* W_master, const float* const* dW, float* const* m,
                        float* const* v, const at_grpo_adam* opt, float* grad_norm,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Bytes of workspace a call needs.  `batch` may be NULL for AT_GRPO_CALL_GROUP_ADVANTAGE; the
 * id extents are ignored for the other calls.  Only sizes are read from `batch` (H, V, n_heads,
 * dtype, n_tok, n_resp); no pointer in it is dereferenced.  Returns 0 on invalid arguments.
 */
size_t at_grpo_workspace_bytes(int32_t which_call, const at_grpo_batch* batch, int32_t n_resp,
                               int32_t n_env, int32_t n_agent, int32_t n_turn);

/* Static description of a status code. */
const char* at_grpo_status_string(int32_t status);

/* Library version, major * 10000 + minor * 100 + patch. */
int32_t at_grpo_version(void);

/*
 * Optional per-kernel timing with HIP events recorded on the call's stream (a measurement aid,
 * off by default; it keeps process-wide state and is not thread-safe).
 *   at_grpo_profile_enable(1) starts recording, (0) stops and drops what was recorded.
 *   at_grpo_profile_read synchronises the recorded events and returns, for kernel class
 *   `which` (0 .. at_grpo_profile_classes()-1), the number of launches and their total
 *   duration in milliseconds since recording started; the name is a static string.
 */
int at_grpo_profile_enable(int32_t on);
int32_t at_grpo_profile_classes(void);
int at_grpo_profile_read(int32_t which, const char** name, int64_t* launches, double* total_ms);

#ifdef __cplusplus
}
#endif
#endif /* AT_GRPO_H_ */
