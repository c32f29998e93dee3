// prune_enumerate_direct: Eq. 3 of Sec. 3.2 evaluated as it is written, without per-token Gram matrices -- for
// every kept set C and token t the difference F'(x_t, C) - F(x_t) = sum_e d_e E_e(x_t) is formed over the hidden
// units (d = Eq. 1 weights of the pruned routing minus those of the full routing: at most 2 k rows) and its
// squares are summed.  It exists to be measured against the Gram path and to cross-check it with different
// arithmetic; it is the better of the two only for a handful of subsets.
//
// One workgroup walks tokens b, b + blocks, ...  Per token: the token's E expert rows are fetched from memory
// once into LDS (so the pass reads Y once, like the Gram pass; the next token's rows are already on their way into
// registers while the current token is scored); thread s works out subset s's routing and leaves the rows and
// coefficients of d in LDS; then the whole workgroup goes through the subsets, each thread covering its share of
// the hidden units, a wavefront reduction per (subset, token) pair.  Pairs whose pruned routing is the full
// routing are skipped and counted: they contribute 0 exactly.
#include <mutex>

#include "common.h"

namespace moep {
namespace {

constexpr int DIR_MAX_SUB = 128;         // subsets (one thread each for the routing, all of them in the main loop)
constexpr int DIR_MAX_K = 4;             // top-k: d has at most 2 k non-zero entries
constexpr int DIR_MAX_ROWS = 2 * DIR_MAX_K;
constexpr int DIR_BLOCKS = 512;          // two workgroups per CU of a 256-CU part (by their LDS at E H = 32768 bf16)

struct DirList {                         // d of one subset for the current token
  int m;                                 // non-zero entries; 0: routing unchanged, nothing to add
  int row[DIR_MAX_ROWS];                 // expert
  float coef[DIR_MAX_ROWS];              // d_e
};

typedef uint32_t bf16x8_bits __attribute__((ext_vector_type(4)));   // 16 bytes: 8 bf16
typedef float f32x4 __attribute__((ext_vector_type(4)));             // 16 bytes: 4 fp32

template <typename V> struct DirVec;
template <> struct DirVec<bf16x8_bits> {
  static constexpr int N = 8;
  static constexpr moep_dtype DT = MOEP_BF16;
  static __device__ void widen(const bf16x8_bits v, float* f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(v[i] << 16);
      f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
    }
  }
};
template <> struct DirVec<f32x4> {
  static constexpr int N = 4;
  static constexpr moep_dtype DT = MOEP_F32;
  static __device__ void widen(const f32x4 v, float* f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = v[i];
  }
};

// The first `count` experts of `allow` in routing order: larger logit first, ties to the lower index.
template <int EMAX>
__device__ uint32_t select_top(const float* l, int E, uint32_t allow, int count, float* first_logit) {
  uint32_t sel = 0;
  *first_logit = 0.f;
#pragma unroll
  for (int j = 0; j < DIR_MAX_K; ++j) {
    if (j >= count) break;
    int best = -1;
    float bl = 0.f;
#pragma unroll
    for (int e = 0; e < EMAX; ++e)
      if (e < E && ((allow >> e) & 1u) && !((sel >> e) & 1u) && (best < 0 || l[e] > bl)) { best = e; bl = l[e]; }
    if (best >= 0) {
      sel |= 1u << best;
      if (j == 0) *first_logit = bl;
    }
  }
  return sel;
}

constexpr int DIR_PREFETCH = 16;         // 16-byte pieces of the next token's rows a thread holds in registers

// A thread's pieces of token t's rows: piece q = chunk q % chunks of expert q / chunks, q = tid, tid + 256, ...
template <typename V>
__device__ __forceinline__ void direct_fetch(V (&held)[DIR_PREFETCH], const V* __restrict__ Y, int64_t t, int64_t T,
                                             int chunks, int total, int tid) {
#pragma unroll
  for (int i = 0; i < DIR_PREFETCH; ++i) {
    const int q = tid + 256 * i < total ? tid + 256 * i : 0;
    held[i] = Y[((int64_t)(q / chunks) * T + t) * chunks + q % chunks];
  }
}

// One thread's share of || sum_i d_i y_i ||^2 for one (subset, token) pair: hidden-unit chunks tid, tid + 256, ...
template <typename V, int MR>
__device__ __forceinline__ float direct_pair(const V* rows, const int* at, const float* d, int chunks, int tid) {
  float acc = 0.f;
  for (int c = tid; c < chunks; c += 256) {
    V v[MR];
#pragma unroll
    for (int i = 0; i < MR; ++i) v[i] = rows[at[i] + c];
    float diff[DirVec<V>::N];
#pragma unroll
    for (int j = 0; j < DirVec<V>::N; ++j) diff[j] = 0.f;
#pragma unroll
    for (int i = 0; i < MR; ++i) {
      float y[DirVec<V>::N];
      DirVec<V>::widen(v[i], y);
#pragma unroll
      for (int j = 0; j < DirVec<V>::N; ++j) diff[j] = fmaf(d[i], y[j], diff[j]);
    }
#pragma unroll
    for (int j = 0; j < DirVec<V>::N; ++j) acc = fmaf(diff[j], diff[j], acc);
  }
  return acc;
}

// EMAX: 8, 16 or 32 >= E.  PREFETCH: a token's rows are at most 256 x DIR_PREFETCH pieces and the next token's
// are held in registers; else the rows are fetched when their token's turn comes.
template <typename V, int EMAX, bool PREFETCH>
__global__ __launch_bounds__(256) void direct_kernel(const float* __restrict__ logits, const V* __restrict__ Y,
                                                     const uint32_t* __restrict__ masks, int64_t T, int E, int H,
                                                     int k, int kk, int n_sub, float* __restrict__ partial,
                                                     uint32_t* __restrict__ partial_cnt) {
  extern __shared__ __align__(16) char smem[];
  const int chunks = H / DirVec<V>::N;                 // 16-byte chunks per row
  const int total = E * chunks;                        // per token: expert e's row of token t sits at Y + (e T + t) chunks
  V* rows = (V*)smem;                                  // [E][chunks]
  DirList* lists = (DirList*)(smem + (((size_t)total * sizeof(V) + 15) & ~(size_t)15));
  float* lossacc = (float*)(lists + DIR_MAX_SUB);      // [4 wavefronts][DIR_MAX_SUB]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 4 * DIR_MAX_SUB; i += 256) lossacc[i] = 0.f;
  const uint32_t my_mask = tid < n_sub ? masks[tid] : 0u;
  const uint32_t all = E == 32 ? 0xffffffffu : (1u << E) - 1u;
  uint32_t same_cnt = 0;
  V held[DIR_PREFETCH];
  if (PREFETCH) direct_fetch(held, Y, blockIdx.x, T, chunks, total, tid);      // gridDim.x <= T
  for (int64_t t = blockIdx.x; t < T; t += gridDim.x) {
    __syncthreads();                                   // the previous token's rows and lists are no longer read
    if (PREFETCH) {
#pragma unroll
      for (int i = 0; i < DIR_PREFETCH; ++i)
        if (tid + 256 * i < total) rows[tid + 256 * i] = held[i];
      // the next token's, in flight while this one is scored (after the last token: this one's again, unused)
      direct_fetch(held, Y, t + gridDim.x < T ? t + gridDim.x : t, T, chunks, total, tid);
    } else {
      for (int q = tid; q < total; q += 256) rows[q] = Y[((int64_t)(q / chunks) * T + t) * chunks + q % chunks];
    }
    // thread s: routing of the full layer and of the layer pruned to subset s, Eq. 1 for both, d = b - a
    if (tid < n_sub) {
      float l[EMAX];
#pragma unroll
      for (int e = 0; e < EMAX; ++e) l[e] = e < E ? logits[t * E + e] : 0.f;
      float first_f, first_p;
      const uint32_t sel_f = select_top<EMAX>(l, E, all, k, &first_f);
      const uint32_t sel_p = select_top<EMAX>(l, E, my_mask, kk, &first_p);
      DirList& L = lists[tid];
      if (sel_p == sel_f) {
        L.m = 0;
        same_cnt += 1;
      } else {
        float wf[EMAX], wp[EMAX], sum_f = 0.f, sum_p = 0.f;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
          wf[e] = ((sel_f >> e) & 1u) ? expf(l[e] - first_f) : 0.f;
          wp[e] = ((sel_p >> e) & 1u) ? expf(l[e] - first_p) : 0.f;
          sum_f += wf[e];
          sum_p += wp[e];
        }
        int m = 0;
#pragma unroll
        for (int e = 0; e < EMAX; ++e)
          if (((sel_f | sel_p) >> e) & 1u) {
            L.row[m] = e * chunks;                     // where the expert's row starts in `rows`
            L.coef[m] = wp[e] / sum_p - wf[e] / sum_f;
            ++m;
          }
        L.m = m;
      }
    }
    __syncthreads();
    for (int s = 0; s < n_sub; ++s) {
      const int m = lists[s].m;                        // the same for every thread
      if (m == 0) continue;
      float d[DIR_MAX_ROWS];
      int at[DIR_MAX_ROWS];
#pragma unroll
      for (int i = 0; i < DIR_MAX_ROWS; ++i) {
        d[i] = i < m ? lists[s].coef[i] : 0.f;
        at[i] = i < m ? lists[s].row[i] : 0;
      }
      // rows beyond m have coefficient 0 and read the first row again: four or eight LDS reads in flight at a time
      float acc = m <= DIR_MAX_ROWS / 2 ? direct_pair<V, DIR_MAX_ROWS / 2>(rows, at, d, chunks, tid)
                                        : direct_pair<V, DIR_MAX_ROWS>(rows, at, d, chunks, tid);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
      if (lane == 0) lossacc[wave * DIR_MAX_SUB + s] += acc;
    }
  }
  __syncthreads();
  if (tid < n_sub) {
    const int64_t o = (int64_t)blockIdx.x * n_sub + tid;
    partial[o] = (lossacc[tid] + lossacc[DIR_MAX_SUB + tid]) + (lossacc[2 * DIR_MAX_SUB + tid] + lossacc[3 * DIR_MAX_SUB + tid]);
    partial_cnt[o] = kk == k ? same_cnt : 0u;
  }
}

// The kernel's dynamic LDS limit is raised to the whole 160 KB once per instantiation and GPU (under a mutex: first
// calls from several host threads are safe; later calls, e.g. under graph capture, only launch).
constexpr int kMaxDevices = 64;
std::mutex g_attr_mu;

template <typename V, int EMAX, bool PREFETCH>
int launch_direct2(const DirectPlan& p, const float* logits, const void* Y, const uint32_t* masks, int kk,
                   float* partial, uint32_t* pcnt, hipStream_t s) {
  static bool raised[kMaxDevices] = {};
  int dev = -1;
  MOEP_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices)
    return fail(MOEP_EUNSUPPORTED, "prune_enumerate_direct: device ordinal %d beyond %d", dev, kMaxDevices - 1);
  {
    std::lock_guard<std::mutex> lk(g_attr_mu);
    if (!raised[dev]) {
      MOEP_HIP(hipFuncSetAttribute((const void*)direct_kernel<V, EMAX, PREFETCH>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
      raised[dev] = true;
    }
  }
  hipLaunchKernelGGL((direct_kernel<V, EMAX, PREFETCH>), dim3((unsigned)p.blocks), dim3(256), p.lds_bytes, s, logits,
                     (const V*)Y, masks, p.T, p.E, p.H, p.k, kk, (int)p.n_sub, partial, pcnt);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

template <typename V, int EMAX>
int launch_direct(const DirectPlan& p, const float* logits, const void* Y, const uint32_t* masks, int kk,
                  float* partial, uint32_t* pcnt, hipStream_t s) {
  const int64_t pieces = (int64_t)p.E * p.H * (int64_t)dtype_size(DirVec<V>::DT) / 16;
  return pieces <= 256 * DIR_PREFETCH ? launch_direct2<V, EMAX, true>(p, logits, Y, masks, kk, partial, pcnt, s)
                                      : launch_direct2<V, EMAX, false>(p, logits, Y, masks, kk, partial, pcnt, s);
}

}  // namespace

int plan_enumerate_direct(int64_t T, int E, int H, int k, int r, moep_dtype dt, DirectPlan* p) {
  const char* who = "prune_enumerate_direct";
  if (k < 1 || k > E) return fail(MOEP_EINVAL, "%s: k=%d out of range [1, E=%d]", who, k, E);
  if (r < 1 || r > E) return fail(MOEP_EINVAL, "%s: r=%d out of range [1, E=%d]", who, r, E);
  if (k > DIR_MAX_K) return fail(MOEP_EUNSUPPORTED, "%s: k=%d above %d", who, k, DIR_MAX_K);
  p->T = T; p->E = E; p->H = H; p->k = k; p->r = r;
  p->n_sub = binomial(E, r);
  if (p->n_sub > DIR_MAX_SUB)
    return fail(MOEP_EUNSUPPORTED, "%s: C(%d,%d) = %lld subsets, at most %d (use prune_enumerate)", who, E, r,
                (long long)p->n_sub, DIR_MAX_SUB);
  const int vec = dt == MOEP_BF16 ? 8 : 4;
  if (H % vec) return fail(MOEP_EUNSUPPORTED, "%s: H=%d must be a multiple of %d", who, H, vec);
  const size_t row_bytes = ((size_t)E * H * dtype_size(dt) + 15) & ~(size_t)15;
  p->lds_bytes = row_bytes + DIR_MAX_SUB * sizeof(DirList) + 4 * DIR_MAX_SUB * sizeof(float);
  if (p->lds_bytes > 160 * 1024)
    return fail(MOEP_EUNSUPPORTED, "%s: the %d rows of a token (%zu bytes) do not fit the LDS", who, E, row_bytes);
  p->blocks = (int)(T < DIR_BLOCKS ? T : DIR_BLOCKS);
  size_t off = 0;
  p->off_masks = off; off += align256((size_t)p->n_sub * sizeof(uint32_t));
  p->off_partial = off; off += align256((size_t)DIR_BLOCKS * p->n_sub * sizeof(float));
  p->off_partial_cnt = off; off += align256((size_t)DIR_BLOCKS * p->n_sub * sizeof(uint32_t));
  p->total = off;
  return MOEP_OK;
}

int launch_enumerate_direct(const DirectPlan& p, const float* logits, const void* Y, moep_dtype dt, float* loss,
                            int32_t* argmin, uint32_t* argmin_mask, int64_t* unaffected, char* ws, hipStream_t s) {
  uint32_t* masks = (uint32_t*)(ws + p.off_masks);
  float* partial = (float*)(ws + p.off_partial);
  uint32_t* pcnt = (uint32_t*)(ws + p.off_partial_cnt);
  const int kk = p.k < p.r ? p.k : p.r;
  if (p.T > 0) {
    if (int st = launch_subset_masks(p.E, p.r, p.n_sub, masks, s)) return st;
    Timed t("direct_gather_weight_reduce", s);
    int st;
    if (dt == MOEP_BF16)
      st = p.E <= 8    ? launch_direct<bf16x8_bits, 8>(p, logits, Y, masks, kk, partial, pcnt, s)
           : p.E <= 16 ? launch_direct<bf16x8_bits, 16>(p, logits, Y, masks, kk, partial, pcnt, s)
                       : launch_direct<bf16x8_bits, 32>(p, logits, Y, masks, kk, partial, pcnt, s);
    else
      st = p.E <= 8    ? launch_direct<f32x4, 8>(p, logits, Y, masks, kk, partial, pcnt, s)
           : p.E <= 16 ? launch_direct<f32x4, 16>(p, logits, Y, masks, kk, partial, pcnt, s)
                       : launch_direct<f32x4, 32>(p, logits, Y, masks, kk, partial, pcnt, s);
    if (st) return st;
  }
  return launch_reduce_argmin(partial, pcnt, p.T > 0 ? p.blocks : 0, p.n_sub, p.E, p.r, loss, argmin, argmin_mask,
                              unaffected, s);
}

}  // namespace moep
