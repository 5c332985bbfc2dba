// Launchers of the LM-head kernels: forward contraction with online-softmax partials, the
// partial combine, and the three backward contractions.  All take device-side token counts, so
// no launch depends on a host read-back.
#pragma once

#include "common.hpp"

namespace atg {

// Geometry of one head pass over a super-chunk of at most TC compacted tokens.
struct HeadGeom {
  int dtype;        // at_grpo_dtype
  int H, V;
  int Vp;           // V rounded up to 64 (k padding of the dZ / W^T buffers)
  int TC;           // tokens per super-chunk (multiple of 256)
  int n_vtiles;     // ceil(V / 256)
  int esize;        // bytes per element of hidden / W / dZ
};

struct HeadChunk {
  const int32_t* idx;   // compacted token rows of this head (device), whole list
  const int32_t* cnt;   // number of entries in idx (device scalar)
  int32_t c0;           // first list position of this super-chunk
};

// part_m / part_s: [n_vtiles][TC] per-(vocabulary tile, token) running max (log2 domain) and
// sum; zy: [TC] target logit.  hidden / W are the caller's tensors.
// part_u: null, or [n_vtiles][TC] partial sums for the entropy monitor (selects the kernel variant).
int launch_head_fwd(const HeadGeom& g, const HeadChunk& ch, const void* hidden, const void* W,
                    const int32_t* token_id, float* part_m, float* part_s, float* part_u, float* zy,
                    hipStream_t s, const int32_t* gate = nullptr);

// logp[row], lse[row] for the rows of this super-chunk (lse may be null).
// With part_u, also entropy[row] = lse - E_p[z].
int launch_lse_combine(const HeadGeom& g, const HeadChunk& ch, const float* part_m,
                       const float* part_s, const float* part_u, const float* zy, float* logp,
                       float* lse, float* entropy, hipStream_t s, const int32_t* gate = nullptr);

// Wt[H][Vp] = W[V][H]^T, zero in the k padding.
int launch_transpose_w(const HeadGeom& g, const void* W, void* Wt, hipStream_t s);

// fp32: hT[H][TC] = (gathered hidden rows of this super-chunk)^T, zero for columns past the count.
// bf16: hT[TC][H] = the gathered rows themselves, zero rows up to the next multiple of 256.
// bf16 with `scale`: row j is multiplied by scale[j] (j counted from the start of the super-chunk).
// bf16 with `perm`: row j is list position perm[j] (and its factor), for j < *live_cnt; zero rows behind.
int launch_gather_transpose_hidden(const HeadGeom& g, const HeadChunk& ch, const void* hidden,
                                   void* hT, hipStream_t s, const float* scale = nullptr,
                                   const int32_t* perm = nullptr, const int32_t* live_cnt = nullptr);

// dZ[TC][Vp] for this super-chunk (element type of hidden); fp32 also fills dZt[V][TC].
int launch_head_dz(const HeadGeom& g, const HeadChunk& ch, const void* hidden, const void* W,
                   const int32_t* token_id, const float* lse, const float* coef, void* dZ, void* dZt,
                   hipStream_t s, const int32_t* gate = nullptr);

// ---- forward and backward from one pass over the logits (bf16) ---------------------------------------
// A `gate` argument of the launchers above and below is a device word: with a non-null gate the kernel
// returns at once while the word is 0 (coef == null in launch_head_dz: dZ = softmax - onehot).
struct CoefArgs;

// c2[j] = log2(e) * z[j][y_j], the reference of the exponentials, for the tokens of the launch.
int launch_ref_logit(const HeadGeom& g, const HeadChunk& ch, const void* hidden, const void* W,
                     const int32_t* token_id, float* c2, hipStream_t s);

// E[j][v] = exp(z[j][v] - c_j) (bf16, [TC][Vp]); part_s[n_vtiles][TC] partial row sums; zy[TC] target logit.
int launch_head_fe(const HeadGeom& g, const HeadChunk& ch, const void* hidden, const void* W,
                   const int32_t* token_id, const float* c2, void* E, float* part_s, float* zy, hipStream_t s);

// logp / lse of the rows; scale[j] = -g_j / S_j; E[j][y_j] = e_y - S_j; raises *gate when a row's sum is
// out of range (that row gets scale 0).
int launch_fe_combine(const HeadGeom& g, const HeadChunk& ch, int head, const float* part_s, const float* c2,
                      const float* zy, const int32_t* token_id, const CoefArgs& ca, float* logp, float* lse,
                      float* scale, void* E, int32_t* gate, hipStream_t s);

// Runs only while *gate != 0: scale[j] = -g_j from logp (E then holds softmax - onehot).
int launch_fallback_scale(const HeadGeom& g, const HeadChunk& ch, int head, const CoefArgs& ca, const float* logp,
                          float* scale, const int32_t* gate, hipStream_t s);

// d_hidden[row] = dZ[j] . Wt^T for the rows of this super-chunk.
// With `scale`, row j of the result is multiplied by scale[j] (j counted from ch.c0).  With `perm` (after
// launch_compact_rows), the first *live_cnt rows of dZ are contracted and row j goes to list position perm[j].
int launch_head_dh(const HeadGeom& g, const HeadChunk& ch, const void* dZ, const void* Wt,
                   void* d_hidden, hipStream_t s, const float* scale = nullptr, const int32_t* perm = nullptr,
                   const int32_t* live_cnt = nullptr);

// Takes the rows with scale[j] == 0 out of a super-chunk of E (bf16, TC <= 32768): rows from the tail are
// copied into their places, so that rows 0 .. *live_cnt - 1 all have a non-zero factor; perm[j] = the list
// position (counted from ch.c0) whose row now sits at j.  holes / movers: scratch of TC entries each;
// *pair_cnt = rows moved.  Deterministic.
int launch_compact_rows(const HeadGeom& g, const HeadChunk& ch, const float* scale, void* E, int32_t* perm,
                        int32_t* holes, int32_t* movers, int32_t* live_cnt, int32_t* pair_cnt, hipStream_t s);

// dW[V][H] (+)= dZ^T . hidden rows.  first_chunk: runs even for an empty list so that dW is defined.
// bf16 with `live_cnt`: only the first *live_cnt rows of the chunk are contracted.
int launch_head_dw(const HeadGeom& g, const HeadChunk& ch, const void* dZ, const void* dZt, const void* hT,
                   float* dW, int accumulate, int first_chunk, hipStream_t s, const int32_t* live_cnt = nullptr);

}  // namespace atg
