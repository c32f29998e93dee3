// An empirical ceiling for the bf16 GEMM kernels: the MFMA stream of gemm_packed_kernel's K loop and nothing
// else.  Same launch shape (one workgroup of 4 wavefronts per compute unit, one wavefront per SIMD), same
// instruction (v_mfma_f32_16x16x32_bf16), same 8 x 8 accumulator tiles per wavefront in 256 AGPRs, same order of
// the MFMAs, two operand register sets used in turn as the double-buffered fragments are -- but no LDS reads,
// no global loads, no barriers, no epilogue.  The operand values are taken from the caller's tensors (the
// layer's activations and weights), because what this part sustains depends on the operand bits: on zeros it
// runs at its nominal peak, on real data the power limit holds the clock well below.
#include <mutex>

#include "common.h"

namespace moep {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void mfma_ceiling_kernel(const bf16x8* __restrict__ a_src, const bf16x8* __restrict__ b_src,
                         float* __restrict__ sink, int steps) {
  bf16x8 fa[2][8], fb[2][8];
  const size_t base = ((size_t)blockIdx.x * 256 + threadIdx.x) * 16;
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) { fa[s][i] = a_src[base + s * 8 + i]; fb[s][i] = b_src[base + s * 8 + i]; }
  f32x4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
  for (int s = 0; s < steps; s += 2) {
#pragma unroll
    for (int slot = 0; slot < 2; ++slot) {
      // (opaque: the fragments count as redefined every step, as in the real loop, which keeps the accumulators in AGPRs)
#pragma unroll
      for (int i = 0; i < 8; ++i) { asm volatile("" : "+v"(fa[slot][i])); asm volatile("" : "+v"(fb[slot][i])); }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
          const int j = (i & 1) ? 7 - jj : jj;
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[slot][j], fa[slot][i], acc[i][j], 0, 0, 0);
        }
    }
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) t += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  sink[blockIdx.x * 256 + threadIdx.x] = t;
}

}  // namespace
}  // namespace moep

using namespace moep;

extern "C" int moep_mfma_ceiling(const void* a_src, const void* b_src, size_t src_bytes, int steps, float* sink,
                                 size_t sink_floats, double* flop_out, void* hip_stream) {
  const char* who = "moep_mfma_ceiling";
  if (!a_src || !b_src || !sink) return fail(MOEP_EINVAL, "%s: NULL pointer", who);
  if (steps < 2 || steps % 2 || steps > (1 << 24)) return fail(MOEP_EINVAL, "%s: steps=%d must be even, 2 .. 2^24", who, steps);
  if (((uintptr_t)a_src | (uintptr_t)b_src) & 15) return fail(MOEP_EUNSUPPORTED, "%s: operands must be 16-byte aligned", who);
  int dev = 0, cus = 0;
  MOEP_HIP(hipGetDevice(&dev));
  MOEP_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  if (cus <= 0) cus = 256;
  const size_t threads = (size_t)cus * 256;
  if (src_bytes < threads * 16 * 16)
    return fail(MOEP_EINVAL, "%s: each operand source must hold %zu bytes, has %zu", who, threads * 256, src_bytes);
  if (sink_floats < threads) return fail(MOEP_EINVAL, "%s: sink must hold %zu floats", who, threads);
  if (flop_out) *flop_out = 2.0 * 128 * 128 * 32 * (double)steps * 4 * cus;   // per wavefront and step: 64 MFMAs of 16x16x32
  hipStream_t s = (hipStream_t)hip_stream;
  Timed t("mfma_ceiling", s);
  hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(cus), dim3(256), 0, s, (const bf16x8*)a_src, (const bf16x8*)b_src,
                     sink, steps);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}
