// Router logits l[t,e] = sum_h x[t,h] Wgate[e,h] (Sec. 3.1), fp32 result.
//
// Bandwidth-bound: x is read once, Wgate (E x H) stays in L1/L2.  bf16 goes through
// router_mfma_kernel below; fp32 storage (and bf16 with H not a multiple of 32) through this kernel: a wavefront takes four
// tokens at a time; lane l owns the h-chunks l, l + 64, ... of every row (16 bytes each), keeps
// 4 x E partial sums and a butterfly of shuffles adds them across the lanes.  The summation
// order for a token depends on nothing but H, so the same token gives the same bits in any batch
// -- moe_expert_outputs and moe_forward_skip rely on that.
#include "common.h"

namespace moep {
namespace {

constexpr int TOK = 4;

template <bool BF16>
struct Chunk;                      // one 16-byte load and its fp32 expansion
template <>
struct Chunk<true> {
  static constexpr int N = 8;
  __device__ static void load(const void* row, int chunk, float (&v)[8]) {
    const uint4 u = ((const uint4*)row)[chunk];
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __builtin_bit_cast(float, w[i] << 16);
      v[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xffff0000u);
    }
  }
};
template <>
struct Chunk<false> {
  static constexpr int N = 4;
  __device__ static void load(const void* row, int chunk, float (&v)[4]) {
    const float4 f = ((const float4*)row)[chunk];
    v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
  }
};

template <bool BF16, int EMAX>
__global__ __launch_bounds__(256) void router_kernel(const void* __restrict__ x,
                                                     const void* __restrict__ Wgate,
                                                     float* __restrict__ logits, int64_t T, int E,
                                                     int H) {
  using C = Chunk<BF16>;
  constexpr int ES = BF16 ? 2 : 4;
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t n_waves = (int64_t)gridDim.x * 4;
  const int chunks = H / C::N;
  const size_t row_bytes = (size_t)H * ES;

  for (int64_t t0 = wave * TOK; t0 < T; t0 += n_waves * TOK) {
    float acc[TOK][EMAX];
#pragma unroll
    for (int i = 0; i < TOK; ++i)
#pragma unroll
      for (int e = 0; e < EMAX; ++e) acc[i][e] = 0.f;

    for (int c = lane; c < chunks; c += 64) {
      float xv[TOK][C::N];
#pragma unroll
      for (int i = 0; i < TOK; ++i) {
        const int64_t t = t0 + i < T ? t0 + i : T - 1;
        C::load((const char*)x + t * row_bytes, c, xv[i]);
      }
#pragma unroll
      for (int e = 0; e < EMAX; ++e) {
        if (e < E) {
          float wv[C::N];
          C::load((const char*)Wgate + e * row_bytes, c, wv);
#pragma unroll
          for (int i = 0; i < TOK; ++i)
#pragma unroll
            for (int j = 0; j < C::N; ++j) acc[i][e] = fmaf(xv[i][j], wv[j], acc[i][e]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < TOK; ++i)
#pragma unroll
      for (int e = 0; e < EMAX; ++e) {
        if (e < E) {
          float v = acc[i][e];
#pragma unroll
          for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
          if (lane == 0 && t0 + i < T) logits[(t0 + i) * E + e] = v;
        }
      }
  }
}

// bf16, E <= 32: the same product on the MFMA units (the fp32 FMAs and the bf16 unpacking of the kernel
// above cost more cycles than reading x does: 0.57 ms for 262144 x 4096 against 0.44 ms here).  A wavefront
// takes 16 tokens; per 32 hidden units one v_mfma_f32_16x16x32_bf16 multiplies the 16 token rows with the
// (at most 16, zero-padded) expert rows of Wgate, which stay in L1/L2 (WIDE, E > 16: a second MFMA takes experts 16 .. 31).  Lane l supplies row l % 16 and
// hidden units 8 (l / 16) .. + 7 of a slice; register v of lane l of the result is token 4 (l / 16) + v,
// expert l % 16.  A token's sum depends on its own row and H only.  (Two tiles per wavefront sharing the
// Wgate fragments, and 1 KB row-wise loads staged through LDS, both measured slower.)
typedef __attribute__((ext_vector_type(8))) __bf16 r_bf16x8;
typedef __attribute__((ext_vector_type(4))) float r_f32x4;

// PACK: the wavefront also writes its 16 rows of x in the blocked operand layout of the packed GEMM (see
// gemm_bf16_packed.hip: tile of 256 rows, slice of 32 hidden units, row p of a block = 64 bytes whose 16-byte chunk c
// sits at position c ^ ((p >> 2) & 3)) -- the registers it feeds the MFMA with are exactly one row group of a block,
// 1 KB of consecutive bytes per store -- so that the expert pass reads x once for both.  Row groups beyond T, up to
// the end of the last tile, are filled with the last row (their products are never stored).
template <bool PACK, bool WIDE>
__global__ __launch_bounds__(256) void router_mfma_kernel(const uint4* __restrict__ x,
                                                          const uint4* __restrict__ Wgate,
                                                          float* __restrict__ logits, int64_t T, int E,
                                                          int H, uint4* __restrict__ xpacked) {
  const int lane = threadIdx.x & 63;
  const int64_t t0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 16;
  if (t0 >= (PACK ? (T + 255) / 256 * 256 : T)) return;
  const int row = lane & 15, kg = lane >> 4;
  const int chunks = H / 8;
  const int64_t t = t0 + row < T ? t0 + row : T - 1;
  const uint4* xp = x + t * chunks + kg;
  // packed destination of this lane's chunk of slice 0; consecutive slices are 1024 chunks (16 KB) apart
  const int p_row = (int)((t0 + row) & 255);
  uint4* const dst = PACK ? xpacked + ((t0 >> 8) * (int64_t)(H / 32)) * 1024 + p_row * 4 + (kg ^ ((p_row >> 2) & 3)) : nullptr;
  const bool w_valid = row < E, w2_valid = WIDE && 16 + row < E;
  const uint4* wp = Wgate + (int64_t)(w_valid ? row : 0) * chunks + kg;
  const uint4* wp2 = Wgate + (int64_t)(w2_valid ? 16 + row : 0) * chunks + kg;
  r_f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = acc0, acc2 = acc0, acc3 = acc0;
  const int steps = H / 32;
  for (int s0 = 0; s0 < steps; s0 += 8) {
    uint4 xv[8], wv[8], wv2[WIDE ? 8 : 1];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool in = s0 + i < steps;
      xv[i] = in ? xp[(s0 + i) * 4] : make_uint4(0, 0, 0, 0);
      wv[i] = (in && w_valid) ? wp[(s0 + i) * 4] : make_uint4(0, 0, 0, 0);
      if (WIDE) wv2[i] = (in && w2_valid) ? wp2[(s0 + i) * 4] : make_uint4(0, 0, 0, 0);
      if (PACK && in) dst[(int64_t)(s0 + i) * 1024] = xv[i];
    }
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
      acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(r_bf16x8, xv[i]),
                                                     __builtin_bit_cast(r_bf16x8, wv[i]), acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(r_bf16x8, xv[i + 1]),
                                                     __builtin_bit_cast(r_bf16x8, wv[i + 1]), acc1, 0, 0, 0);
      if (WIDE) {
        acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(r_bf16x8, xv[i]),
                                                       __builtin_bit_cast(r_bf16x8, wv2[i]), acc2, 0, 0, 0);
        acc3 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(r_bf16x8, xv[i + 1]),
                                                       __builtin_bit_cast(r_bf16x8, wv2[i + 1]), acc3, 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int64_t tt = t0 + 4 * kg + v;
    if (tt < T && row < E) logits[tt * E + row] = acc0[v] + acc1[v];
    if (WIDE && tt < T && 16 + row < E) logits[tt * E + 16 + row] = acc2[v] + acc3[v];
  }
}

bool mfma_router_applies(int E, int H) { return E <= 32 && H % 32 == 0; }

template <bool PACK>
void launch_mfma(const void* x, const void* Wgate, int64_t T, int E, int H, float* logits, void* xpacked,
                 int64_t blocks, hipStream_t s) {
  if (E > 16)
    hipLaunchKernelGGL((router_mfma_kernel<PACK, true>), dim3((unsigned)blocks), dim3(256), 0, s, (const uint4*)x,
                       (const uint4*)Wgate, logits, T, E, H, (uint4*)xpacked);
  else
    hipLaunchKernelGGL((router_mfma_kernel<PACK, false>), dim3((unsigned)blocks), dim3(256), 0, s, (const uint4*)x,
                       (const uint4*)Wgate, logits, T, E, H, (uint4*)xpacked);
}

template <bool BF16>
int launch_t(const void* x, const void* Wgate, int64_t T, int E, int H, float* logits, hipStream_t s) {
  if (BF16 && mfma_router_applies(E, H)) {
    const int64_t blocks = ceil_div(T, 64);
    if (blocks < ((int64_t)1 << 31)) {
      launch_mfma<false>(x, Wgate, T, E, H, logits, nullptr, blocks, s);
      MOEP_HIP(hipGetLastError());
      return MOEP_OK;
    }
  }
  const int64_t groups = ceil_div(T, TOK);
  const unsigned blocks = (unsigned)(ceil_div(groups, 4) < 16384 ? ceil_div(groups, 4) : 16384);
  if (E <= 8) hipLaunchKernelGGL((router_kernel<BF16, 8>), dim3(blocks), dim3(256), 0, s, x, Wgate, logits, T, E, H);
  else if (E <= 16) hipLaunchKernelGGL((router_kernel<BF16, 16>), dim3(blocks), dim3(256), 0, s, x, Wgate, logits, T, E, H);
  else hipLaunchKernelGGL((router_kernel<BF16, 32>), dim3(blocks), dim3(256), 0, s, x, Wgate, logits, T, E, H);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

}  // namespace

int launch_router(const void* x, const void* Wgate, int64_t T, int E, int H, moep_dtype dt,
                  float* logits, hipStream_t s) {
  if (T <= 0) return MOEP_OK;
  if (H % (dt == MOEP_BF16 ? 8 : 4)) return fail(MOEP_EUNSUPPORTED, "router: H=%d not a multiple of the 16-byte chunk", H);
  if (((uintptr_t)x | (uintptr_t)Wgate) & 15) return fail(MOEP_EUNSUPPORTED, "router: x and Wgate must be 16-byte aligned");
  Timed t("router_logits", s);
  return dt == MOEP_BF16 ? launch_t<true>(x, Wgate, T, E, H, logits, s)
                         : launch_t<false>(x, Wgate, T, E, H, logits, s);
}

// bf16: router logits and the packed copy of x in one pass over x.  Returns MOEP_EUNSUPPORTED without launching
// anything when the shape has no fused kernel (the caller then runs the router and the packing separately).
int launch_router_and_pack_x(const void* x, const void* Wgate, int64_t T, int E, int H, float* logits, void* xpacked,
                             hipStream_t s) {
  if (T <= 0) return MOEP_OK;
  const int64_t blocks = ceil_div(ceil_div(T, 256) * 256, 64);
  if (!mfma_router_applies(E, H) || H % 64 || blocks >= ((int64_t)1 << 31)) return MOEP_EUNSUPPORTED;
  if (((uintptr_t)x | (uintptr_t)Wgate | (uintptr_t)xpacked) & 15)
    return fail(MOEP_EUNSUPPORTED, "router: x, Wgate and the packed copy of x must be 16-byte aligned");
  Timed t("router_logits_pack_x", s);
  launch_mfma<true>(x, Wgate, T, E, H, logits, xpacked, blocks, s);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

}  // namespace moep
