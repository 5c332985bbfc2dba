// Update of the head weights after the policy-loss backward (gfx950).
//
// Alg. 1, Phase 2 ends with "update policy m"; App. C.1 fixes how: gradient clipping at 1.0, Adam
// with learning rate 1e-6 and weight decay 0.01.  Two streaming passes over the head's gradient:
//   1. the squared L2 norm of all heads' gradients taken together (block partials, then one
//      fixed-order reduction in fp64: deterministic), from which the clip factor
//      min(1, max_norm / (norm + 1e-6));
//   2. one fused pass per element: scale the gradient, update both Adam moments, step the fp32
//      master weight and write the bf16 copy the head kernels read.
// Both are bound by HBM: pass 1 reads 4 bytes per parameter, pass 2 reads 16 and writes 14 (12 for
// fp32 heads, which have no separate low-precision copy).
#include "common.hpp"

namespace atg {

namespace {

constexpr int kNormBlocks = 1024;   // partial sums per head

struct UpdatePtrs {
  const float* g[kMaxHeads];
  float* m[kMaxHeads];
  float* v[kMaxHeads];
  float* master[kMaxHeads];   // fp32 weights that are stepped
  bf16_t* low[kMaxHeads];     // bf16 copy (null for fp32 heads)
};

struct AdamConst {
  float beta1, beta2, one_minus_beta1, one_minus_beta2;
  float eps;
  float step_size;      // lr / (1 - beta1^step)
  float inv_sqrt_bc2;   // 1 / sqrt(1 - beta2^step)
  float lr_wd;          // lr * weight_decay   (decoupled form)
  float wd;             // weight_decay        (coupled form)
  int decoupled;
};

__global__ __launch_bounds__(256) void k_grad_sqnorm(UpdatePtrs P, int64_t n4, float* __restrict__ partial) {
  __shared__ float red[4];
  const float4* __restrict__ g = reinterpret_cast<const float4*>(P.g[blockIdx.y]);
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n4; i += stride) {
    const float4 x = g[i];
    a0 = fmaf(x.x, x.x, a0);
    a1 = fmaf(x.y, x.y, a1);
    a2 = fmaf(x.z, x.z, a2);
    a3 = fmaf(x.w, x.w, a3);
  }
  const float s = block_sum_256((a0 + a1) + (a2 + a3), red);
  if (threadIdx.x == 0) partial[blockIdx.y * gridDim.x + blockIdx.x] = s;
}

// out[0] = norm over all heads, out[1] = clip factor
__global__ __launch_bounds__(1024) void k_grad_norm_final(const float* __restrict__ partial, int count,
                                                          float max_norm, float* __restrict__ out) {
  __shared__ double red[1024];
  double s = 0.0;
  for (int i = threadIdx.x; i < count; i += 1024) s += static_cast<double>(partial[i]);
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const float norm = static_cast<float>(sqrt(red[0]));
    float coef = 1.f;
    if (max_norm > 0.f) coef = fminf(1.f, max_norm / (norm + 1e-6f));
    out[0] = norm;
    out[1] = coef;
  }
}

__device__ __forceinline__ float adam_one(float g, float& m, float& v, float w, const AdamConst& c) {
  if (!c.decoupled) g = fmaf(c.wd, w, g);
  m = fmaf(c.beta1, m, c.one_minus_beta1 * g);
  v = fmaf(c.beta2, v, c.one_minus_beta2 * g * g);
  const float denom = fmaf(sqrtf(v), c.inv_sqrt_bc2, c.eps);
  // both small terms are summed before they meet w, so the decay is not lost below w's last bit
  float upd = c.step_size * m / denom;
  if (c.decoupled) upd = fmaf(c.lr_wd, w, upd);
  return w - upd;
}

template <bool LOW>
__global__ __launch_bounds__(256) void k_adam(UpdatePtrs P, int64_t n4, AdamConst c,
                                              const float* __restrict__ norm_coef) {
  const int h = blockIdx.y;
  const float coef = norm_coef[1];
  const float4* __restrict__ g4 = reinterpret_cast<const float4*>(P.g[h]);
  float4* __restrict__ m4 = reinterpret_cast<float4*>(P.m[h]);
  float4* __restrict__ v4 = reinterpret_cast<float4*>(P.v[h]);
  float4* __restrict__ w4 = reinterpret_cast<float4*>(P.master[h]);
  uint2* __restrict__ l4 = reinterpret_cast<uint2*>(P.low[h]);
  const int64_t stride = static_cast<int64_t>(gridDim.x) * 256;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n4; i += stride) {
    const float4 g = g4[i];
    float4 m = m4[i], v = v4[i], w = w4[i];
    w.x = adam_one(g.x * coef, m.x, v.x, w.x, c);
    w.y = adam_one(g.y * coef, m.y, v.y, w.y, c);
    w.z = adam_one(g.z * coef, m.z, v.z, w.z, c);
    w.w = adam_one(g.w * coef, m.w, v.w, w.w, c);
    m4[i] = m;
    v4[i] = v;
    w4[i] = w;
    if (LOW) l4[i] = make_uint2(pack_bf16x2(w.x, w.y), pack_bf16x2(w.z, w.w));
  }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

size_t head_update_workspace() {
  WsAlloc ws(nullptr);
  ws.take<int32_t>(64);
  ws.take<float>(static_cast<size_t>(kMaxHeads) * kNormBlocks);
  return ws.bytes();
}

}  // namespace atg

using namespace atg;

extern "C" int at_grpo_head_update(int32_t dtype, int32_t H, int32_t V, int32_t n_heads, void* const* W,
                                   float* const* W_master, const float* const* dW, float* const* m,
                                   float* const* v, const at_grpo_adam* opt, float* grad_norm,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!W || !dW || !m || !v || !opt || !grad_norm) return AT_GRPO_EINVAL;
  if (dtype != AT_GRPO_F32 && dtype != AT_GRPO_BF16) return AT_GRPO_EUNSUPPORTED;
  if (H <= 0 || V <= 0 || n_heads < 1 || n_heads > kMaxHeads) return AT_GRPO_EINVAL;
  if (H % 4 != 0) return AT_GRPO_EUNSUPPORTED;
  if (dtype == AT_GRPO_BF16 && !W_master) return AT_GRPO_EINVAL;
  if (opt->step < 1 || !(opt->lr >= 0.f) || !(opt->beta1 >= 0.f && opt->beta1 < 1.f) ||
      !(opt->beta2 >= 0.f && opt->beta2 < 1.f) || !(opt->eps > 0.f) || !(opt->weight_decay >= 0.f) ||
      !(opt->max_grad_norm >= 0.f))
    return AT_GRPO_EINVAL;
  UpdatePtrs P{};
  for (int h = 0; h < n_heads; ++h) {
    P.g[h] = dW[h];
    P.m[h] = m[h];
    P.v[h] = v[h];
    P.master[h] = dtype == AT_GRPO_BF16 ? W_master[h] : static_cast<float*>(W[h]);
    P.low[h] = dtype == AT_GRPO_BF16 ? static_cast<bf16_t*>(W[h]) : nullptr;
    if (!P.g[h] || !P.m[h] || !P.v[h] || !P.master[h] || !W[h]) return AT_GRPO_EINVAL;
    if (!aligned16(P.g[h]) || !aligned16(P.m[h]) || !aligned16(P.v[h]) || !aligned16(P.master[h]) ||
        !aligned16(W[h]))
      return AT_GRPO_EINVAL;
  }
  WsAlloc ws(workspace);
  ws.take<int32_t>(64);   // error word slot, kept for the common workspace layout
  float* partial = ws.take<float>(static_cast<size_t>(kMaxHeads) * kNormBlocks);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < ws.bytes())
    return AT_GRPO_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  const int64_t n4 = static_cast<int64_t>(V) * H / 4;
  const double bc1 = 1.0 - pow(static_cast<double>(opt->beta1), opt->step);
  const double bc2 = 1.0 - pow(static_cast<double>(opt->beta2), opt->step);
  AdamConst c;
  c.beta1 = opt->beta1;
  c.beta2 = opt->beta2;
  c.one_minus_beta1 = static_cast<float>(1.0 - static_cast<double>(opt->beta1));
  c.one_minus_beta2 = static_cast<float>(1.0 - static_cast<double>(opt->beta2));
  c.eps = opt->eps;
  c.step_size = static_cast<float>(static_cast<double>(opt->lr) / bc1);
  c.inv_sqrt_bc2 = static_cast<float>(1.0 / sqrt(bc2));
  c.lr_wd = static_cast<float>(static_cast<double>(opt->lr) * opt->weight_decay);
  c.wd = opt->weight_decay;
  c.decoupled = opt->decoupled != 0;

  {
    ProfScope ps(PROF_GRAD_NORM, s);
    hipLaunchKernelGGL(k_grad_sqnorm, dim3(kNormBlocks, n_heads), dim3(256), 0, s, P, n4, partial);
    ATG_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_grad_norm_final, dim3(1), dim3(1024), 0, s, partial, n_heads * kNormBlocks,
                       opt->max_grad_norm, grad_norm);
    ATG_LAUNCH_CHECK();
  }
  {
    ProfScope ps(PROF_ADAM, s);
    const int64_t want = ceil_div(n4, 256 * 4);
    const unsigned blocks = static_cast<unsigned>(want > 8192 ? 8192 : (want < 1 ? 1 : want));
    if (dtype == AT_GRPO_BF16)
      hipLaunchKernelGGL(k_adam<true>, dim3(blocks, n_heads), dim3(256), 0, s, P, n4, c, grad_norm);
    else
      hipLaunchKernelGGL(k_adam<false>, dim3(blocks, n_heads), dim3(256), 0, s, P, n4, c, grad_norm);
    ATG_LAUNCH_CHECK();
  }
  return AT_GRPO_OK;
}
