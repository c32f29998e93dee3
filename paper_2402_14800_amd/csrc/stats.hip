// Expert-selection statistics over a calibration set (baselines of Sec. 4.1; appendix on expert
// selection tendency): count[e] = tokens whose top-k contains e, co[i][j] = tokens whose top-k
// contains both i and j, and the activation-frequency baseline's kept set (the r most selected
// experts, lower index first on equal counts).  Integer work throughout: per-block LDS tables,
// then integer atomics, so the result does not depend on the order of execution.
#include "common.h"

namespace moep {
namespace {

constexpr int SB_THREADS = 256;

__global__ __launch_bounds__(SB_THREADS) void stats_zero_kernel(unsigned long long* count, unsigned long long* co, int E) {
  for (int i = threadIdx.x; i < E * E; i += SB_THREADS) co[i] = 0;
  if ((int)threadIdx.x < E) count[threadIdx.x] = 0;
}

__global__ __launch_bounds__(SB_THREADS) void stats_kernel(const float* __restrict__ logits, int64_t T, int E, int k,
                                                          unsigned long long* __restrict__ count,
                                                          unsigned long long* __restrict__ co) {
  __shared__ unsigned int tab[32][33];       // [i][j], j < 32; column 32 unused padding
  for (int i = threadIdx.x; i < 32 * 33; i += SB_THREADS) (&tab[0][0])[i] = 0;
  __syncthreads();
  for (int64_t t = (int64_t)blockIdx.x * SB_THREADS + threadIdx.x; t < T; t += (int64_t)gridDim.x * SB_THREADS) {
    const float* l = logits + t * E;
    float v[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) v[e] = e < E ? l[e] : 0.f;
    uint32_t mask = 0;                       // expert e is in the top-k iff fewer than k experts come before it
#pragma unroll
    for (int e = 0; e < 32; ++e) {
      int before = 0;
#pragma unroll
      for (int f = 0; f < 32; ++f)
        if (f < E) before += (v[f] > v[e]) || (v[f] == v[e] && f < e);
      if (e < E && before < k) mask |= 1u << e;
    }
    for (uint32_t mi = mask; mi; mi &= mi - 1) {
      const int i = __builtin_ctz(mi);
      for (uint32_t mj = mask; mj; mj &= mj - 1) atomicAdd(&tab[i][__builtin_ctz(mj)], 1u);
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < E * E; idx += SB_THREADS) {
    const int i = idx / E, j = idx - i * E;
    const unsigned int c = tab[i][j];
    if (c) {
      atomicAdd(&co[idx], (unsigned long long)c);
      if (i == j) atomicAdd(&count[i], (unsigned long long)c);
    }
  }
}

__global__ void frequency_mask_kernel(const unsigned long long* __restrict__ count, int E, int r, uint32_t* mask_out) {
  if (threadIdx.x || blockIdx.x) return;
  uint32_t mask = 0;
  for (int e = 0; e < E; ++e) {              // kept iff fewer than r experts are ranked before e
    int before = 0;
    for (int f = 0; f < E; ++f) before += (count[f] > count[e]) || (count[f] == count[e] && f < e);
    if (before < r) mask |= 1u << e;
  }
  *mask_out = mask;
}

}  // namespace

int launch_selection_stats(const float* logits, int64_t T, int E, int k, int r, int64_t* count, int64_t* co,
                           uint32_t* freq_mask, hipStream_t s) {
  Timed t("selection_stats", s);
  hipLaunchKernelGGL(stats_zero_kernel, dim3(1), dim3(SB_THREADS), 0, s, (unsigned long long*)count,
                     (unsigned long long*)co, E);
  if (T > 0) {
    const int64_t want = ceil_div(T, SB_THREADS);
    const unsigned blocks = (unsigned)(want < 2048 ? want : 2048);
    hipLaunchKernelGGL(stats_kernel, dim3(blocks), dim3(SB_THREADS), 0, s, logits, T, E, k,
                       (unsigned long long*)count, (unsigned long long*)co);
  }
  if (freq_mask)
    hipLaunchKernelGGL(frequency_mask_kernel, dim3(1), dim3(64), 0, s, (const unsigned long long*)count, E, r, freq_mask);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

}  // namespace moep
