// fp32 GEMM (storage type MOEP_F32): C = epilogue(A B^T), A [M,K], B [N,K], plain FMA arithmetic.
// Serves the small fp32 configuration; the layout of arguments, epilogues and the grouped tile
// map (256-row M tiles) are those of the bf16 kernel.  A workgroup of 256 threads owns a 64 x 64
// tile (4 x 4 outputs per thread) and walks K in steps of 16 through LDS.
#include "common.h"

namespace moep {
namespace {

constexpr int TM = 64, TN = 64, TK = 16, THREADS = 256;

struct FArgs {
  const float* A; const float* B0; const float* B1;
  const int32_t* a_rows;
  float* C;
  const float* row_scale;
  const int32_t* tile_expert; const int32_t* tile_row0; const int32_t* seg_end;
  int64_t M, lda, ldc, b_expert_stride;
  int N, K;
};

template <int EPI>
__global__ __launch_bounds__(THREADS) void gemm_f32_kernel(FArgs p) {
  __shared__ float sA[TK][TM + 4];
  __shared__ float sB[TK][TN + 4];
  __shared__ float sU[EPI == EPI_SWIGLU ? TK : 1][TN + 4];

  // blockIdx.x walks 64-row sub-tiles; in grouped mode four of them share one 256-row map entry.
  int64_t row0, row_end;
  const float* B0 = p.B0;
  const float* B1 = p.B1;
  if (p.tile_expert) {
    const int t = blockIdx.x >> 2;
    const int e = p.tile_expert[t];
    if (e < 0) return;
    row0 = (int64_t)p.tile_row0[t] + (blockIdx.x & 3) * TM;
    row_end = p.seg_end[e];
    if (row0 >= row_end) return;
    B0 += (int64_t)e * p.b_expert_stride;
    if (EPI == EPI_SWIGLU) B1 += (int64_t)e * p.b_expert_stride;
  } else {
    row0 = (int64_t)blockIdx.x * TM;
    row_end = p.M;
  }
  const int n0 = blockIdx.y * TN;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;          // outputs rows ty*4.., cols tx*4..

  // staging: thread loads 4 consecutive k of one row
  const int lr = tid >> 2;                         // 0..63
  const int lk = (tid & 3) * 4;                    // 0,4,8,12
  int64_t ar = row0 + lr;
  if (ar >= row_end) ar = row_end - 1;
  const int64_t asrc = p.a_rows ? (int64_t)p.a_rows[ar] : ar;
  const float* ap = p.A + asrc * p.lda + lk;
  int bn = n0 + lr;
  if (bn >= p.N) bn = p.N - 1;
  const float* bp = B0 + (int64_t)bn * p.K + lk;
  const float* up = EPI == EPI_SWIGLU ? B1 + (int64_t)bn * p.K + lk : nullptr;

  float acc[4][4] = {}, accu[4][4] = {};
  for (int k0 = 0; k0 < p.K; k0 += TK) {
    float4 va = make_float4(0.f, 0.f, 0.f, 0.f), vb = va, vu = va;
    if (k0 + lk < p.K) {                           // K is a multiple of 4
      va = *(const float4*)(ap + k0);
      vb = *(const float4*)(bp + k0);
      if (EPI == EPI_SWIGLU) vu = *(const float4*)(up + k0);
    }
    sA[lk + 0][lr] = va.x; sA[lk + 1][lr] = va.y; sA[lk + 2][lr] = va.z; sA[lk + 3][lr] = va.w;
    sB[lk + 0][lr] = vb.x; sB[lk + 1][lr] = vb.y; sB[lk + 2][lr] = vb.z; sB[lk + 3][lr] = vb.w;
    if (EPI == EPI_SWIGLU) {
      sU[lk + 0][lr] = vu.x; sU[lk + 1][lr] = vu.y; sU[lk + 2][lr] = vu.z; sU[lk + 3][lr] = vu.w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], b[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sA[kk][ty * 4 + i]; b[i] = sB[kk][tx * 4 + i]; }
      if (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int i = 0; i < 4; ++i) u[i] = sU[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
          if (EPI == EPI_SWIGLU) accu[i][j] = fmaf(a[i], u[j], accu[i][j]);
        }
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t r = row0 + ty * 4 + i;
    if (r >= row_end) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= p.N) continue;
      float v = acc[i][j];
      if (EPI == EPI_SWIGLU) v = v / (1.0f + expf(-v)) * accu[i][j];
      if (EPI == EPI_ROWSCALE_F32) v *= p.row_scale[r];
      p.C[r * p.ldc + n] = v;
    }
  }
}

}  // namespace

int launch_gemm_f32(const GemmArgs& g, hipStream_t s, const char* name) {
  if (g.K % 4 || g.K <= 0 || g.lda % 4) return fail(MOEP_EUNSUPPORTED, "%s: K=%d and lda must be multiples of 4", name, g.K);
  if (g.M <= 0 || g.N <= 0) return MOEP_OK;
  FArgs f;
  f.A = (const float*)g.A; f.B0 = (const float*)g.B0; f.B1 = (const float*)g.B1;
  f.a_rows = g.a_rows; f.C = (float*)g.C; f.row_scale = g.row_scale;
  f.tile_expert = g.tile_expert; f.tile_row0 = g.tile_row0; f.seg_end = g.seg_end;
  f.M = g.M; f.lda = g.lda; f.ldc = g.ldc; f.b_expert_stride = g.b_expert_stride;
  f.N = g.N; f.K = g.K;
  const int64_t m_tiles = g.tile_expert ? g.max_m_tiles * (GEMM_BM / TM) : ceil_div(g.M, TM);
  const int64_t n_tiles = ceil_div(g.N, TN);
  if (m_tiles > 2147483647LL || n_tiles > 65535) return fail(MOEP_EUNSUPPORTED, "%s: too many tiles", name);
  dim3 grid((unsigned)m_tiles, (unsigned)n_tiles);
  Timed t(name, s);
  switch (g.epilogue) {
    case EPI_STORE: hipLaunchKernelGGL(gemm_f32_kernel<EPI_STORE>, grid, dim3(THREADS), 0, s, f); break;
    case EPI_SWIGLU: hipLaunchKernelGGL(gemm_f32_kernel<EPI_SWIGLU>, grid, dim3(THREADS), 0, s, f); break;
    case EPI_ROWSCALE_F32: hipLaunchKernelGGL(gemm_f32_kernel<EPI_ROWSCALE_F32>, grid, dim3(THREADS), 0, s, f); break;
    default: return fail(MOEP_EINVAL, "%s: unknown epilogue %d", name, g.epilogue);
  }
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

}  // namespace moep
