/*
 * abi_client.c -- a plain C99 caller of libat_grpo.so.
 *
 * Shows (and lets the tests check) that the boundary is usable without Python or C++: it includes
 * at_grpo.h as C, fills the at_grpo_batch struct the way a C compiler lays it out, owns every
 * buffer through the HIP C API and reads results back itself.
 *
 *   abi_client <input.txt> <output.txt>
 *
 * input.txt, whitespace separated:
 *   group_advantage R n_env n_agent n_turn eps_std ddof norm
 *       then R lines:  env_id agent_id turn_id reward
 *   policy_loss_fwd H V n_tok R eps_low eps_high agg          (fp32, one head, packed layout)
 *       then (R+1) cu_seqlens, R advantages, n_tok lines "token_id old_logp",
 *       n_tok*H hidden values, V*H head weights
 * Floats are written with %a (hex) on both sides, so no bit is lost in the text files.
 * output.txt: one value per line in the order the sections are named there.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "at_grpo.h"

#define HIP_OK(expr)                                                        \
  do {                                                                      \
    hipError_t e_ = (expr);                                                 \
    if (e_ != hipSuccess) {                                                 \
      fprintf(stderr, "%s: %s\n", #expr, hipGetErrorString(e_));            \
      return 3;                                                             \
    }                                                                       \
  } while (0)

#define AT_OK(expr)                                                         \
  do {                                                                      \
    int s_ = (expr);                                                        \
    if (s_ != AT_GRPO_OK) {                                                 \
      fprintf(stderr, "%s: %s\n", #expr, at_grpo_status_string(s_));        \
      return 4;                                                             \
    }                                                                       \
  } while (0)

static void* to_device(const void* host, size_t bytes) {
  void* d = NULL;
  if (hipMalloc(&d, bytes ? bytes : 4) != hipSuccess) return NULL;
  if (bytes && hipMemcpy(d, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
  return d;
}

static int run_group_advantage(FILE* in, FILE* out) {
  int R, E, N, T, ddof, norm;
  float eps;
  if (fscanf(in, "%d %d %d %d %a %d %d", &R, &E, &N, &T, &eps, &ddof, &norm) != 7 || R <= 0) return 2;
  int32_t* ids = (int32_t*)malloc(sizeof(int32_t) * 3 * (size_t)R);
  float* reward = (float*)malloc(sizeof(float) * (size_t)R);
  for (int r = 0; r < R; ++r)
    if (fscanf(in, "%d %d %d %a", &ids[r], &ids[R + r], &ids[2 * R + r], &reward[r]) != 4) return 2;
  const int gmax = R < E * N * T ? R : E * N * T;
  int32_t* d_ids = (int32_t*)to_device(ids, sizeof(int32_t) * 3 * (size_t)R);
  float* d_reward = (float*)to_device(reward, sizeof(float) * (size_t)R);
  int32_t *d_gid, *d_ng, *d_off, *d_perm;
  float *d_adv, *d_mean, *d_std;
  HIP_OK(hipMalloc((void**)&d_gid, sizeof(int32_t) * (size_t)R));
  HIP_OK(hipMalloc((void**)&d_ng, sizeof(int32_t)));
  HIP_OK(hipMalloc((void**)&d_off, sizeof(int32_t) * (size_t)(gmax + 1)));
  HIP_OK(hipMalloc((void**)&d_perm, sizeof(int32_t) * (size_t)R));
  HIP_OK(hipMalloc((void**)&d_adv, sizeof(float) * (size_t)R));
  HIP_OK(hipMalloc((void**)&d_mean, sizeof(float) * (size_t)gmax));
  HIP_OK(hipMalloc((void**)&d_std, sizeof(float) * (size_t)gmax));
  const size_t ws_bytes = at_grpo_workspace_bytes(AT_GRPO_CALL_GROUP_ADVANTAGE, NULL, R, E, N, T);
  void* ws = NULL;
  if (!d_ids || !d_reward || ws_bytes == 0) return 3;
  HIP_OK(hipMalloc(&ws, ws_bytes));
  AT_OK(at_grpo_group_advantage(R, E, N, T, d_ids, d_ids + R, d_ids + 2 * R, d_reward, eps, ddof, norm, d_gid,
                                d_ng, d_off, d_perm, d_adv, d_mean, d_std, ws, ws_bytes, NULL));
  HIP_OK(hipDeviceSynchronize());
  int32_t G = 0, err = 0;
  HIP_OK(hipMemcpy(&G, d_ng, sizeof(G), hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(&err, ws, sizeof(err), hipMemcpyDeviceToHost));
  int32_t* h_i = (int32_t*)malloc(sizeof(int32_t) * (size_t)(2 * R + gmax + 1));
  float* h_f = (float*)malloc(sizeof(float) * (size_t)(R + 2 * gmax));
  HIP_OK(hipMemcpy(h_i, d_gid, sizeof(int32_t) * (size_t)R, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(h_i + R, d_perm, sizeof(int32_t) * (size_t)R, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(h_i + 2 * R, d_off, sizeof(int32_t) * (size_t)(G + 1), hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(h_f, d_adv, sizeof(float) * (size_t)R, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(h_f + R, d_mean, sizeof(float) * (size_t)G, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(h_f + R + gmax, d_std, sizeof(float) * (size_t)G, hipMemcpyDeviceToHost));
  fprintf(out, "error_word %d\nn_groups %d\n", err, G);
  fprintf(out, "group_id\n");
  for (int r = 0; r < R; ++r) fprintf(out, "%d\n", h_i[r]);
  fprintf(out, "perm\n");
  for (int r = 0; r < R; ++r) fprintf(out, "%d\n", h_i[R + r]);
  fprintf(out, "seg_offsets\n");
  for (int g = 0; g <= G; ++g) fprintf(out, "%d\n", h_i[2 * R + g]);
  fprintf(out, "adv\n");
  for (int r = 0; r < R; ++r) fprintf(out, "%a\n", h_f[r]);
  fprintf(out, "group_mean\n");
  for (int g = 0; g < G; ++g) fprintf(out, "%a\n", h_f[R + g]);
  fprintf(out, "group_std\n");
  for (int g = 0; g < G; ++g) fprintf(out, "%a\n", h_f[R + gmax + g]);
  return 0;
}

static int run_policy_loss_fwd(FILE* in, FILE* out) {
  int H, V, n_tok, R, agg;
  float eps_low, eps_high;
  if (fscanf(in, "%d %d %d %d %a %a %d", &H, &V, &n_tok, &R, &eps_low, &eps_high, &agg) != 7) return 2;
  if (H <= 0 || V <= 0 || n_tok <= 0 || R <= 0) return 2;
  int64_t* cu = (int64_t*)malloc(sizeof(int64_t) * (size_t)(R + 1));
  float* adv = (float*)malloc(sizeof(float) * (size_t)R);
  int32_t* tok = (int32_t*)malloc(sizeof(int32_t) * (size_t)n_tok);
  float* old_logp = (float*)malloc(sizeof(float) * (size_t)n_tok);
  float* hidden = (float*)malloc(sizeof(float) * (size_t)n_tok * (size_t)H);
  float* W = (float*)malloc(sizeof(float) * (size_t)V * (size_t)H);
  for (int r = 0; r <= R; ++r) {
    long long v;
    if (fscanf(in, "%lld", &v) != 1) return 2;
    cu[r] = v;
  }
  for (int r = 0; r < R; ++r)
    if (fscanf(in, "%a", &adv[r]) != 1) return 2;
  for (int t = 0; t < n_tok; ++t)
    if (fscanf(in, "%d %a", &tok[t], &old_logp[t]) != 2) return 2;
  for (size_t k = 0; k < (size_t)n_tok * (size_t)H; ++k)
    if (fscanf(in, "%a", &hidden[k]) != 1) return 2;
  for (size_t k = 0; k < (size_t)V * (size_t)H; ++k)
    if (fscanf(in, "%a", &W[k]) != 1) return 2;

  const void* d_W = to_device(W, sizeof(float) * (size_t)V * (size_t)H);
  const void* heads[1];
  heads[0] = d_W;
  at_grpo_batch b;
  memset(&b, 0, sizeof(b));
  b.dtype = AT_GRPO_F32;
  b.H = H;
  b.V = V;
  b.n_heads = 1;
  b.n_tok = n_tok;
  b.n_resp = R;
  b.n_agent = 0;
  b.cu_seqlens = (const int64_t*)to_device(cu, sizeof(int64_t) * (size_t)(R + 1));
  b.hidden = to_device(hidden, sizeof(float) * (size_t)n_tok * (size_t)H);
  b.W = heads;
  b.token_id = (const int32_t*)to_device(tok, sizeof(int32_t) * (size_t)n_tok);
  b.mask = NULL;
  b.resp_agent = NULL;
  b.head_of_agent = NULL;
  float* d_old = (float*)to_device(old_logp, sizeof(float) * (size_t)n_tok);
  float* d_adv = (float*)to_device(adv, sizeof(float) * (size_t)R);
  if (!d_W || !b.cu_seqlens || !b.hidden || !b.token_id || !d_old || !d_adv) return 3;
  float *d_loss, *d_logp, *d_lse;
  uint8_t* d_clip;
  int32_t* d_nvalid;
  HIP_OK(hipMalloc((void**)&d_loss, sizeof(float)));
  HIP_OK(hipMalloc((void**)&d_logp, sizeof(float) * (size_t)n_tok));
  HIP_OK(hipMalloc((void**)&d_lse, sizeof(float) * (size_t)n_tok));
  HIP_OK(hipMalloc((void**)&d_clip, (size_t)n_tok));
  HIP_OK(hipMalloc((void**)&d_nvalid, sizeof(int32_t)));
  const size_t ws_bytes = at_grpo_workspace_bytes(AT_GRPO_CALL_POLICY_LOSS_FWD, &b, 0, 0, 0, 0);
  if (ws_bytes == 0) return 3;
  void* ws = NULL;
  HIP_OK(hipMalloc(&ws, ws_bytes));
  AT_OK(at_grpo_policy_loss_fwd(&b, d_old, d_adv, eps_low, eps_high, agg, d_loss, d_logp, d_lse, d_clip, d_nvalid,
                                ws, ws_bytes, NULL));
  HIP_OK(hipDeviceSynchronize());
  float loss = 0.f;
  int32_t nvalid = 0, err = 0;
  HIP_OK(hipMemcpy(&loss, d_loss, sizeof(loss), hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(&nvalid, d_nvalid, sizeof(nvalid), hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(&err, ws, sizeof(err), hipMemcpyDeviceToHost));
  float* h_logp = (float*)malloc(sizeof(float) * (size_t)n_tok);
  uint8_t* h_clip = (uint8_t*)malloc((size_t)n_tok);
  HIP_OK(hipMemcpy(h_logp, d_logp, sizeof(float) * (size_t)n_tok, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(h_clip, d_clip, (size_t)n_tok, hipMemcpyDeviceToHost));
  fprintf(out, "error_word %d\nn_valid %d\nloss %a\n", err, nvalid, loss);
  fprintf(out, "logp\n");
  for (int t = 0; t < n_tok; ++t) fprintf(out, "%a\n", h_logp[t]);
  fprintf(out, "clip_mask\n");
  for (int t = 0; t < n_tok; ++t) fprintf(out, "%d\n", (int)h_clip[t]);
  return 0;
}

int main(int argc, char** argv) {
  if (argc != 3) {
    fprintf(stderr, "usage: %s input.txt output.txt\n", argv[0]);
    return 2;
  }
  FILE* in = fopen(argv[1], "r");
  FILE* out = fopen(argv[2], "w");
  if (!in || !out) return 2;
  char what[64];
  if (fscanf(in, "%63s", what) != 1) return 2;
  int rc = 2;
  if (strcmp(what, "group_advantage") == 0) rc = run_group_advantage(in, out);
  if (strcmp(what, "policy_loss_fwd") == 0) rc = run_policy_loss_fwd(in, out);
  fprintf(out, "version %d\n", at_grpo_version());
  fclose(out);
  fclose(in);
  return rc;
}
