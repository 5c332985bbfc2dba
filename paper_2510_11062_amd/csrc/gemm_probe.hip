// Measurement aid: the tile loops of the head kernels run as plain bf16 GEMMs, without any epilogue work,
// so that the loop itself can be compared with a vendor GEMM on the shapes the library uses.
//
//   gemm_probe <variant> M N K
//     nt    C[m][n] = sum_k A[m][k] B[n][k]   gemm_tile of gemm_core.hpp: the loop of the forward, dZ and
//                                             dHidden kernels (256 x 256 tile, 8 wavefronts, 128-byte k-steps)
//     km    C[m][n] = sum_k A[k][m] B[k][n]   gemm_tile_kmajor: the k-major loop (dW)
//     nt4, km4                                the same loops with 4 wavefronts of 128 x 128 per workgroup
//                                             (the layout the dHidden and dW kernels use)
//     wg2   as nt, with a different layout that was tried and rejected: 4-wavefront workgroups on 256 x 128
//           tiles, 64-byte k-steps in three LDS stages of 24 KiB, two workgroups resident per compute unit (so
//           that one workgroup's epilogue could overlap the other's MFMAs)
// M, N multiples of 256, K a multiple of 64 (wg2: (K / 32) % 3 == 1).  Prints the time per launch, the
// achieved TFLOP/s and the shader clock (cycle counter against the 100 MHz wall clock) after checking 600
// sampled outputs of a 512 x 512 corner against fp64 sums on the host.  Not part of the library.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "gemm_core.hpp"

#define CHECK(x)                                                                       \
  do {                                                                                 \
    hipError_t e_ = (x);                                                               \
    if (e_ != hipSuccess) {                                                            \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);            \
      exit(1);                                                                         \
    }                                                                                  \
  } while (0)

namespace {

using namespace atg;

constexpr size_t kClockSlot = (size_t{16} << 20) - 1;   // float index in C where workgroup 0 leaves the clock

template <int IB, int JB>
__device__ __forceinline__ float sum_acc(floatx16 (&acc)[IB][JB]) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < IB; ++i)
#pragma unroll
    for (int j = 0; j < JB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][j][r];
  return s;
}

template <bool KMAJOR, typename G>
__global__ __launch_bounds__(G::kThreads) void k_probe(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                        float* __restrict__ C, int M, int N, int K, int write_c) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const long long clk0 = clock64(), wall0 = wall_clock64();
  const TileOrder ord{M / kTile, N / kTile, 8};
  const TileCoordT<G> tc;
  float sink = 0.f;
  for (int t = logical_workgroup(); t < ord.total(); t += gridDim.x) {
    int ta, tb;
    ord.decode(t, &ta, &tb);
    floatx16 acc[G::kIB][G::kJB];
    if (KMAJOR) {
      gemm_tile_kmajor<G>(acc, reinterpret_cast<const char*>(A + ta * kTile), static_cast<size_t>(M) * 2, 31,
                       reinterpret_cast<const char*>(B + tb * kTile), static_cast<size_t>(N) * 2, 31, K / kKmRows, smem);
    } else {
      const size_t row_bytes = static_cast<size_t>(K) * 2;
      gemm_tile<bf16_t, G>(
          acc,
          [&](int row) { return reinterpret_cast<const char*>(A) + static_cast<size_t>(ta * kTile + row) * row_bytes; },
          [&](int row) { return reinterpret_cast<const char*>(B) + static_cast<size_t>(tb * kTile + row) * row_bytes; },
          static_cast<int>(row_bytes / kStepBytes), smem);
    }
    if (write_c) {
#pragma unroll
      for (int i = 0; i < G::kIB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
#pragma unroll
          for (int j = 0; j < G::kJB; ++j)
            C[static_cast<size_t>(ta * kTile + tc.a_row(i, r)) * N + tb * kTile + tc.b_row(j)] = acc[i][j][r];
    } else {
      sink += sum_acc(acc);
    }
  }
  if (!write_c && sink == 12345.678f) C[threadIdx.x] = sink;   // keeps the contraction alive
  if (!write_c && blockIdx.x == 0 && threadIdx.x == 0)
    C[kClockSlot] = static_cast<float>(clock64() - clk0) / static_cast<float>(wall_clock64() - wall0) * 100.f;
}

// ---- the rejected two-workgroups-per-compute-unit layout ------------------------------------------------
namespace wg2 {
constexpr int kTA = 256, kTB = 128;            // tile rows of A and of B
constexpr int kStep = 64;                      // bytes of k per row per step
constexpr int kLdsA = kTA * kStep, kLdsB = kTB * kStep, kStageBytes = kLdsA + kLdsB, kLds = 3 * kStageBytes;
constexpr int kLdA = 4, kLdB = 2, kLd = kLdA + kLdB;   // direct loads per wavefront per step

__device__ __forceinline__ int swz4(int row) { return (((row >> 2) & 1) << 1) | ((row >> 3) & 1); }
template <int N>
__device__ __forceinline__ void wait_vm(/* vmcnt(N), lgkmcnt(0) */) {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | 0x70 | ((N >> 4) << 14));
}

struct Ops {
  floatx16 (&acc)[kIB][kJB];
  const char* (&ap)[kLdA];
  const char* (&bp)[kLdB];
  const int (&rd_a)[kIB];
  const int (&rd_b)[kJB];
  const int (&sw_a)[kIB];
  const int (&sw_b)[kJB];
  uint32_t lds_a, lds_b;
  int half;
  uint4 fa[2][kIB], fb[2][kJB];
  __device__ __forceinline__ void mm(int f, int n) { Mma<bf16_t>::run(fa[f][n / kJB], fb[f][n % kJB], acc[n / kJB][n % kJB]); }
  __device__ __forceinline__ void rd(const char* stage, int ks, int f, int n) {
    const int c = (ks << 1) | half;
    if (n < kIB) fa[f][n] = *reinterpret_cast<const uint4*>(stage + rd_a[n] + ((c ^ sw_a[n]) << 4));
    else fb[f][n - kIB] = *reinterpret_cast<const uint4*>(stage + rd_b[n - kIB] + ((c ^ sw_b[n - kIB]) << 4));
  }
  __device__ __forceinline__ void ld(int stage, int d) {
    if (d < kLdA) {
      direct_load16(ap[d], lds_a + stage * kStageBytes + d * 1024);
      ap[d] += kStep;
    } else {
      direct_load16(bp[d - kLdA], lds_b + stage * kStageBytes + (d - kLdA) * 1024);
      bp[d - kLdA] += kStep;
    }
  }
};

// step kt on stage s0 = kt % 3: the loads of step kt+2 (second half) and kt+3 (first half) are requested,
// step kt+1 must have landed at the barrier in the middle
template <int s0, bool LAST>
__device__ __forceinline__ void step(Ops& ops, char* smem) {
  constexpr int s1 = (s0 + 1) % 3, s2 = (s0 + 2) % 3;
#pragma unroll
  for (int n = 0; n < 8; ++n) {
    ops.mm(0, n);
    ATG_PIN();
    if (n < 6) {
      ops.rd(smem + s0 * kStageBytes, 1, 1, n);
      ATG_PIN();
    }
    if (!LAST && (n == 1 || n == 4 || n == 6)) {
      ops.ld(s2, 3 + (n == 1 ? 0 : n == 4 ? 1 : 2));
      ATG_PIN();
    }
  }
  if (LAST) wait_vm<0>(); else wait_vm<kLd>();
  __builtin_amdgcn_s_barrier();
  ATG_PIN();
#pragma unroll
  for (int n = 0; n < 8; ++n) {
    ops.mm(1, n);
    ATG_PIN();
    if (!LAST && n < 6) {
      ops.rd(smem + s1 * kStageBytes, 0, 0, n);
      ATG_PIN();
    }
    if (!LAST && (n == 1 || n == 4 || n == 6)) {
      ops.ld(s0, n == 1 ? 0 : n == 4 ? 1 : 2);
      ATG_PIN();
    }
  }
}

__global__ __launch_bounds__(256, 2) void k_probe(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                  float* __restrict__ C, int M, int N, int K, int write_c) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const long long clk0 = clock64(), wall0 = wall_clock64();
  const TileOrder ord{M / kTA, N / kTB, 8};
  const int nk = K * 2 / kStep;                      // (nk % 3 == 1): whole rounds of three stages, then one step
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t row_bytes = static_cast<size_t>(K) * 2;
  float sink = 0.f;
  for (int t = logical_workgroup(); t < ord.total(); t += gridDim.x) {
    int ta, tb;
    ord.decode(t, &ta, &tb);
    floatx16 acc[kIB][kJB];
#pragma unroll
    for (int i = 0; i < kIB; ++i)
#pragma unroll
      for (int j = 0; j < kJB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const char* ap[kLdA];
    const char* bp[kLdB];
#pragma unroll
    for (int q = 0; q < kLdA; ++q) {
      const int row = wave * 64 + q * 16 + (lane >> 2);
      ap[q] = reinterpret_cast<const char*>(A) + static_cast<size_t>(ta * kTA + row) * row_bytes + (((lane & 3) ^ swz4(row)) << 4);
    }
#pragma unroll
    for (int q = 0; q < kLdB; ++q) {
      const int row = wave * 32 + q * 16 + (lane >> 2);
      bp[q] = reinterpret_cast<const char*>(B) + static_cast<size_t>(tb * kTB + row) * row_bytes + (((lane & 3) ^ swz4(row)) << 4);
    }
    int rd_a[kIB], rd_b[kJB], sw_a[kIB], sw_b[kJB];
#pragma unroll
    for (int i = 0; i < kIB; ++i) {
      const int ra = wave * 64 + i * 32 + (lane & 31);
      rd_a[i] = ra * kStep;
      sw_a[i] = swz4(ra);
    }
#pragma unroll
    for (int j = 0; j < kJB; ++j) {
      const int rb = j * 32 + (lane & 31);
      rd_b[j] = kLdsA + rb * kStep;
      sw_b[j] = swz4(rb);
    }
    const uint32_t base = lds_address(smem);
    Ops ops{acc, ap, bp, rd_a, rd_b, sw_a, sw_b,
            static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(base + wave * 64 * kStep)),
            static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(base + kLdsA + wave * 32 * kStep)), lane >> 5, {}, {}};
    // steps 0 and 1 in full and the first half of step 2; the rows are padded on the host so that the three
    // steps requested past the end of a row stay inside the allocation
#pragma unroll
    for (int d = 0; d < kLd; ++d) ops.ld(0, d);
#pragma unroll
    for (int d = 0; d < kLd; ++d) ops.ld(1, d);
#pragma unroll
    for (int d = 0; d < 3; ++d) ops.ld(2, d);
    wait_vm<kLd + 3>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int n = 0; n < 6; ++n) ops.rd(smem, 0, 0, n);
    for (int kt = 0; kt + 3 < nk; kt += 3) {
      step<0, false>(ops, smem);
      step<1, false>(ops, smem);
      step<2, false>(ops, smem);
    }
    step<0, true>(ops, smem);
    if (write_c) {
#pragma unroll
      for (int i = 0; i < kIB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = ta * kTA + wave * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
#pragma unroll
          for (int j = 0; j < kJB; ++j) C[static_cast<size_t>(m) * N + tb * kTB + j * 32 + (lane & 31)] = acc[i][j][r];
        }
    } else {
      sink += sum_acc(acc);
    }
    __builtin_amdgcn_s_barrier();   // all wavefronts are past their last LDS read before the next tile's loads
  }
  if (!write_c && sink == 12345.678f) C[threadIdx.x] = sink;
  if (!write_c && blockIdx.x == 0 && threadIdx.x == 0)
    C[kClockSlot] = static_cast<float>(clock64() - clk0) / static_cast<float>(wall_clock64() - wall0) * 100.f;
}
}  // namespace wg2

uint16_t f2bf(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fff + ((u >> 16) & 1);
  return static_cast<uint16_t>(u >> 16);
}
float bf2f(uint16_t b) {
  const uint32_t u = static_cast<uint32_t>(b) << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

typedef void (*kern_t)(const bf16_t*, const bf16_t*, float*, int, int, int, int);

}  // namespace

int main(int argc, char** argv) {
  if (argc < 5) {
    printf("usage: gemm_probe nt|km|wg2 M N K\n");
    return 2;
  }
  const char* variant = argv[1];
  const int M = atoi(argv[2]), N = atoi(argv[3]), K = atoi(argv[4]);
  const bool four = !strcmp(variant, "nt4") || !strcmp(variant, "km4");
  const bool km = !strcmp(variant, "km") || !strcmp(variant, "km4"), two = !strcmp(variant, "wg2");
  if (!km && !two && strcmp(variant, "nt") && strcmp(variant, "nt4")) { printf("unknown variant\n"); return 2; }
  if (M % 256 || N % 256 || K % (two ? 32 : 64) || M < 512 || N < 512 || K < 64 || (two && (K / 32) % 3 != 1)) {
    printf("unsupported shape\n");
    return 2;
  }
  // A is [M][K] (nt, wg2) or [K][M] (km); B likewise.  4 KiB of padding behind each operand.
  std::vector<uint16_t> hA(static_cast<size_t>(M) * K), hB(static_cast<size_t>(N) * K);
  uint32_t s = 12345;
  auto rnd = [&]() { s = s * 1664525u + 1013904223u; return ((s >> 8) & 0xffff) / 65536.0f - 0.5f; };
  for (auto& x : hA) x = f2bf(rnd());
  for (auto& x : hB) x = f2bf(rnd());
  bf16_t *dA, *dB;
  float* dC;
  CHECK(hipMalloc(&dA, hA.size() * 2 + 4096));
  CHECK(hipMalloc(&dB, hB.size() * 2 + 4096));
  CHECK(hipMalloc(&dC, size_t{64} << 20));
  CHECK(hipMemcpy(dA, hA.data(), hA.size() * 2, hipMemcpyHostToDevice));
  CHECK(hipMemcpy(dB, hB.data(), hB.size() * 2, hipMemcpyHostToDevice));
  kern_t kern = two ? wg2::k_probe
                    : four ? (km ? k_probe<true, G4> : k_probe<false, G4>)
                           : (km ? k_probe<true, G8> : k_probe<false, G8>);
  const int threads = two ? 256 : (four ? G4::kThreads : G8::kThreads), lds = two ? wg2::kLds : kLdsBytes, grid = two ? 512 : 256;
  CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  {
    // correctness on the 512 x 512 corner (full K); for km the corner is taken from operands of 512 columns
    const int m = 512, n = 512;
    bf16_t *cA = dA, *cB = dB;
    std::vector<uint16_t> sA, sB;
    if (km) {   // repack the first 512 columns so that the row stride is 512
      sA.resize(static_cast<size_t>(K) * m);
      sB.resize(static_cast<size_t>(K) * n);
      for (int k = 0; k < K; ++k) {
        memcpy(&sA[static_cast<size_t>(k) * m], &hA[static_cast<size_t>(k) * M], m * 2);
        memcpy(&sB[static_cast<size_t>(k) * n], &hB[static_cast<size_t>(k) * N], n * 2);
      }
      CHECK(hipMalloc(&cA, sA.size() * 2));
      CHECK(hipMalloc(&cB, sB.size() * 2));
      CHECK(hipMemcpy(cA, sA.data(), sA.size() * 2, hipMemcpyHostToDevice));
      CHECK(hipMemcpy(cB, sB.data(), sB.size() * 2, hipMemcpyHostToDevice));
    }
    CHECK(hipMemset(dC, 0, static_cast<size_t>(m) * n * 4));
    hipLaunchKernelGGL(kern, dim3(8), dim3(threads), lds, 0, cA, cB, dC, m, n, K, 1);
    CHECK(hipDeviceSynchronize());
    std::vector<float> hC(static_cast<size_t>(m) * n);
    CHECK(hipMemcpy(hC.data(), dC, hC.size() * 4, hipMemcpyDeviceToHost));
    double maxerr = 0;
    for (int q = 0; q < 600; ++q) {
      const int i = (q * 131) % m, j = (q * 977 + 13) % n;
      double ref = 0;
      for (int k = 0; k < K; ++k)
        ref += km ? static_cast<double>(bf2f(hA[static_cast<size_t>(k) * M + i])) * bf2f(hB[static_cast<size_t>(k) * N + j])
                  : static_cast<double>(bf2f(hA[static_cast<size_t>(i) * K + k])) * bf2f(hB[static_cast<size_t>(j) * K + k]);
      maxerr = fmax(maxerr, fabs(ref - hC[static_cast<size_t>(i) * n + j]));
    }
    if (km) {
      CHECK(hipFree(cA));
      CHECK(hipFree(cB));
    }
    if (!(maxerr < 1e-3 * sqrt(static_cast<double>(K)))) {
      printf("%s: WRONG RESULT, max abs err %.3e\n", variant, maxerr);
      return 1;
    }
    printf("%s check: max abs err %.3e on 600 sampled outputs\n", variant, maxerr);
  }
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  for (int it = 0; it < 2; ++it) hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), lds, 0, dA, dB, dC, M, N, K, 0);
  CHECK(hipDeviceSynchronize());
  const int iters = 5;
  CHECK(hipEventRecord(e0));
  for (int it = 0; it < iters; ++it) hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), lds, 0, dA, dB, dC, M, N, K, 0);
  CHECK(hipEventRecord(e1));
  CHECK(hipDeviceSynchronize());
  float ms = 0.f, mhz = 0.f;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  ms /= iters;
  CHECK(hipMemcpy(&mhz, dC + kClockSlot, 4, hipMemcpyDeviceToHost));
  printf("{\"variant\": \"%s\", \"M\": %d, \"N\": %d, \"K\": %d, \"ms\": %.4f, \"tflops\": %.1f, \"shader_clock_mhz\": %.0f}\n",
         variant, M, N, K, ms, 2.0 * M * N * K / ms / 1e9, mhz);
  return 0;
}
