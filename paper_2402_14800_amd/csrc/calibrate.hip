// Calibration of the skipping threshold (Sec. 3.3; appendix on experiment details): beta is the
// median over the calibration tokens of w_e1 / w_e0 = exp(l_e1 - l_e0), e0 and e1 being the token's
// top-2 experts (among the kept ones).  exp is monotone, so the two middle order statistics of
// delta = l_e1 - l_e0 (fp32, the same subtraction the routing kernel thresholds) are selected
// exactly by a most-significant-digit radix select on the order-preserving integer image of the
// floats, and beta = (exp(delta_lo) + exp(delta_hi)) / 2 is formed in fp64 at the very end.
//
//   keys     one thread per token: top-2 (ties -> lower index), delta, key; block 0 also clears
//            the histograms (a kernel rather than a memset so that the call can be graph-captured)
//   hist     4 passes of 8 bits: count the keys that match the digits chosen so far, separately
//            for the lower and the upper median rank (integer atomics only: order-independent)
//   choose   one block: find the digit whose bucket holds the wanted rank, narrow the rank
//   finish   turn the two keys back into floats and write beta
#include <cmath>

#include "common.h"

namespace moep {
namespace {

constexpr int CB = 256;

struct SelectState {          // per wanted rank q in {0, 1}
  uint32_t prefix[2];         // digits chosen so far, in place
  uint32_t rem[2];            // rank still to find inside the matching keys
};

__device__ __forceinline__ uint32_t float_to_key(float f) {     // ascending floats -> ascending keys
  const uint32_t u = __builtin_bit_cast(uint32_t, f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __builtin_bit_cast(float, u);
}

__global__ __launch_bounds__(CB) void keys_kernel(const float* __restrict__ logits, int64_t T, int E,
                                                  uint32_t kept, uint32_t* __restrict__ keys,
                                                  uint32_t* __restrict__ hist, SelectState* state) {
  if (blockIdx.x == 0) {
    for (int i = threadIdx.x; i < 4 * 2 * 256; i += CB) hist[i] = 0;
    if (threadIdx.x == 0) {
      state->prefix[0] = state->prefix[1] = 0;
      state->rem[0] = (uint32_t)((T - 1) / 2);
      state->rem[1] = (uint32_t)(T / 2);
    }
  }
  const int64_t t = (int64_t)blockIdx.x * CB + threadIdx.x;
  if (t >= T) return;
  const float* l = logits + t * E;
  int e0 = -1, e1 = -1;
  float l0 = 0.f, l1 = 0.f;
  for (int e = 0; e < E; ++e) {
    if (!((kept >> e) & 1u)) continue;
    const float v = l[e];
    if (e0 < 0 || v > l0) { l1 = l0; e1 = e0; l0 = v; e0 = e; }
    else if (e1 < 0 || v > l1) { l1 = v; e1 = e; }
  }
  keys[t] = float_to_key(l1 - l0);
}

__global__ __launch_bounds__(CB) void hist_kernel(const uint32_t* __restrict__ keys, int64_t T, int pass,
                                                  const SelectState* __restrict__ state,
                                                  uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[2][256];
  h[0][threadIdx.x] = 0;
  h[1][threadIdx.x] = 0;
  __syncthreads();
  const int shift = 24 - 8 * pass;
  const uint32_t high = pass == 0 ? 0u : (0xffffffffu << (shift + 8));   // digits already chosen
  const uint32_t p0 = state->prefix[0], p1 = state->prefix[1];
  for (int64_t i = (int64_t)blockIdx.x * CB + threadIdx.x; i < T; i += (int64_t)gridDim.x * CB) {
    const uint32_t k = keys[i];
    const uint32_t d = (k >> shift) & 255u;
    if ((k & high) == p0) atomicAdd(&h[0][d], 1u);
    if ((k & high) == p1) atomicAdd(&h[1][d], 1u);
  }
  __syncthreads();
  uint32_t* g = hist + (size_t)pass * 512;
  if (h[0][threadIdx.x]) atomicAdd(&g[threadIdx.x], h[0][threadIdx.x]);
  if (h[1][threadIdx.x]) atomicAdd(&g[256 + threadIdx.x], h[1][threadIdx.x]);
}

__global__ __launch_bounds__(64) void choose_kernel(const uint32_t* __restrict__ hist, int pass,
                                                    SelectState* state, float* __restrict__ beta_out) {
  const int q = threadIdx.x;
  if (q < 2) {
    const uint32_t* g = hist + (size_t)pass * 512 + q * 256;
    uint32_t rem = state->rem[q], run = 0;
    int d = 0;
    for (; d < 255; ++d) {              // the wanted key is in the first bucket whose running count exceeds rem
      const uint32_t c = g[d];
      if (run + c > rem) break;
      run += c;
    }
    state->prefix[q] |= (uint32_t)d << (24 - 8 * pass);
    state->rem[q] = rem - run;
  }
  if (pass == 3) {
    __syncthreads();
    if (threadIdx.x == 0) {
      const double lo = exp((double)key_to_float(state->prefix[0]));
      const double hi = exp((double)key_to_float(state->prefix[1]));
      *beta_out = (float)(0.5 * (lo + hi));
    }
  }
}

}  // namespace

size_t calibrate_workspace_bytes(int64_t T) {
  return align256((size_t)T * 4) + align256(4 * 2 * 256 * 4) + align256(sizeof(SelectState));
}

int launch_calibrate_beta(const float* logits, int64_t T, int E, uint32_t kept_mask, float* beta_out,
                          char* ws, hipStream_t s) {
  uint32_t* keys = (uint32_t*)ws;
  uint32_t* hist = (uint32_t*)(ws + align256((size_t)T * 4));
  SelectState* state = (SelectState*)((char*)hist + align256(4 * 2 * 256 * 4));
  const int64_t n_blocks = ceil_div(T, CB);
  const unsigned hist_blocks = (unsigned)(n_blocks < 1024 ? n_blocks : 1024);
  Timed t("skip_calibrate_beta", s);
  hipLaunchKernelGGL(keys_kernel, dim3((unsigned)n_blocks), dim3(CB), 0, s, logits, T, E, kept_mask, keys,
                     hist, state);
  for (int pass = 0; pass < 4; ++pass) {
    hipLaunchKernelGGL(hist_kernel, dim3(hist_blocks), dim3(CB), 0, s, keys, T, pass, state, hist);
    hipLaunchKernelGGL(choose_kernel, dim3(1), dim3(64), 0, s, hist, pass, state, beta_out);
  }
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

}  // namespace moep
