// Dynamic skipping, top-2 (Sec. 3.3; output per App. A.2): routing, dispatch and combine.
// The expert FFNs themselves are the grouped GEMMs (see gemm_bf16_packed.hip / gemm_f32.hip).
//
//   route    per token: top-2 experts by logit among the kept experts (ties -> lower index), delta = l_e1 - l_e0 in fp32,
//            skip iff delta < theta = fp32(ln beta) (theta = -inf for beta = 0), weights
//            a0 = 1 / (1 + rho), a1 = rho / (1 + rho), rho = exp(delta); a0 = 1 when skipped.
//            Also counts, per block of 256 tokens, the rows each expert receives.
//   scan     turns the counts into each (block, expert)'s first slot, each expert's segment end,
//            and the map from 256-row M tiles to (expert, first row) that the grouped GEMMs walk
//            (entry [max_tiles] of the expert list holds the number of tiles in use).
//   scatter  writes slot -> token and slot -> weight lists and token -> slot positions.  Within an
//            expert's segment the rows are in ascending token order, so the result is reproducible.
//   combine  out[t] = slot_out[pos0] (+ slot_out[pos1] unless skipped); the down projection has
//            already multiplied each slot by its weight.  No atomics anywhere on this path.
//
// The *_topk kernels are the same pipeline for the generalised rule of the theory appendix: each
// token keeps the top-i* of its top-k experts, i* = min { i : sum_{m>i} w_m <= beta sum_{m<=k} w_m },
// decided in fp64 on the fp32 logits (tail sums accumulated from the smallest weight upwards), and
// the kept weights are renormalised over those i*.
#include <cmath>

#include "common.h"

namespace moep {
namespace {

constexpr int RB = 256;     // tokens per routing block

__global__ __launch_bounds__(RB) void route_kernel(const float* __restrict__ logits, int64_t T,
                                                   int E, uint32_t kept, float theta, uint8_t* __restrict__ skip_mask,
                                                   int32_t* __restrict__ top2,
                                                   float* __restrict__ tw, int32_t* __restrict__ counts) {
  __shared__ int cnt[32];
  if (threadIdx.x < 32) cnt[threadIdx.x] = 0;
  __syncthreads();
  const int64_t t = (int64_t)blockIdx.x * RB + threadIdx.x;
  if (t < T) {
    const float* l = logits + t * E;
    int e0 = -1, e1 = -1;
    float l0 = -INFINITY, l1 = -INFINITY;
    for (int e = 0; e < E; ++e) {          // strict comparisons: the lower index wins a tie
      if (!((kept >> e) & 1u)) continue;   // a removed expert and its routing weight are gone
      const float v = l[e];
      if (e0 < 0 || v > l0) { l1 = l0; e1 = e0; l0 = v; e0 = e; }
      else if (e1 < 0 || v > l1) { l1 = v; e1 = e; }
    }
    const float delta = l1 - l0;
    const bool skip = delta < theta;
    const float rho = expf(delta);
    const float a0 = skip ? 1.0f : 1.0f / (1.0f + rho);
    const float a1 = skip ? 0.0f : rho / (1.0f + rho);
    skip_mask[t] = skip ? 1 : 0;
    top2[2 * t] = e0;
    top2[2 * t + 1] = e1;
    tw[2 * t] = a0;
    tw[2 * t + 1] = a1;
    atomicAdd(&cnt[e0], 1);
    if (!skip) atomicAdd(&cnt[e1], 1);
  }
  __syncthreads();
  if ((int)threadIdx.x < E) counts[(int64_t)blockIdx.x * E + threadIdx.x] = cnt[threadIdx.x];
}

// seg_end holds 2 E + 1 ints: the E segment ends, then the index of each expert's first tile (E + 1 entries,
// the last one being the number of tiles in use).
__global__ __launch_bounds__(256) void scan_kernel(int32_t* __restrict__ counts, int64_t n_blocks,
                                                   int E, int32_t* __restrict__ seg_end,
                                                   int32_t* __restrict__ tile_expert,
                                                   int32_t* __restrict__ tile_row0, int max_tiles) {
  __shared__ int total[32], begin[33];
  __shared__ int n_tiles;
  const int e = threadIdx.x;
  if (e < E) {
    int s = 0;
    for (int64_t b = 0; b < n_blocks; ++b) s += counts[b * E + e];
    total[e] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < E; ++i) { begin[i] = run; run += total[i]; }
    begin[E] = run;
    int idx = 0;
    for (int i = 0; i < E; ++i) {
      seg_end[E + i] = idx;
      for (int row = begin[i]; row < begin[i + 1] && idx < max_tiles; row += GEMM_BM) {
        tile_expert[idx] = i;
        tile_row0[idx] = row;
        ++idx;
      }
    }
    seg_end[2 * E] = idx;
    n_tiles = idx;
    tile_expert[max_tiles] = idx;          // number of tiles in use, read by the grouped GEMMs
  }
  __syncthreads();
  if (e < E) {
    int run = begin[e];
    for (int64_t b = 0; b < n_blocks; ++b) {
      const int c = counts[b * E + e];
      counts[b * E + e] = run;
      run += c;
    }
    seg_end[e] = run;
  }
  for (int i = n_tiles + threadIdx.x; i < max_tiles; i += blockDim.x) {
    tile_expert[i] = -1;
    tile_row0[i] = 0;
  }
}

// The order in which a grouped GEMM launch walks its tiles.  The launch gives every XCD a contiguous run of this
// list; within a run, 32 consecutive entries are in flight together and share operand panels through the XCD's L2.
// Entries are grouped per EXPERT: group_m consecutive M tiles of one expert, walked along N (all group_m tiles of
// one N tile, then the next N tile), so that the tiles in flight share the same few weight panels; an expert's last
// group may be smaller.  Entry = (M tile << 12) | N tile.
__global__ __launch_bounds__(256) void order_kernel(const int32_t* __restrict__ expert_first, int E, int n_tiles,
                                                    int group_m, uint32_t* __restrict__ order) {
  __shared__ int first[33];
  if ((int)threadIdx.x <= E) first[threadIdx.x] = expert_first[threadIdx.x];
  __syncthreads();
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= (int64_t)first[E] * n_tiles) return;
  int e = 0;
  while (e + 1 < E && (int64_t)first[e + 1] * n_tiles <= q) ++e;
  const int64_t qe = q - (int64_t)first[e] * n_tiles;
  const int c = first[e + 1] - first[e];
  const int64_t gsz = (int64_t)group_m * n_tiles;
  const int g = (int)(qe / gsz);
  const int first_m = g * group_m;
  const int gm = c - first_m < group_m ? c - first_m : group_m;
  const int in_group = (int)(qe - g * gsz);
  const int tn = in_group / gm, m = first_m + in_group % gm;
  order[q] = ((uint32_t)(first[e] + m) << 12) | (uint32_t)tn;
}

__global__ __launch_bounds__(RB) void scatter_kernel(const int32_t* __restrict__ top2,
                                                     const float* __restrict__ tw,
                                                     const uint8_t* __restrict__ skip_mask,
                                                     const int32_t* __restrict__ base, int64_t T,
                                                     int E, int32_t* __restrict__ slot_token,
                                                     float* __restrict__ slot_scale,
                                                     int32_t* __restrict__ slot_dest,
                                                     int32_t* __restrict__ pos) {
  __shared__ int wave_cnt[RB / 64][32];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t t = (int64_t)blockIdx.x * RB + threadIdx.x;
  const bool live = t < T;
  const int e0 = live ? top2[2 * t] : -1;
  const int e1 = (live && !skip_mask[t]) ? top2[2 * t + 1] : -1;
  const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  int rank0 = 0, rank1 = 0;
  for (int e = 0; e < E; ++e) {
    const unsigned long long b0 = __ballot(e0 == e), b1 = __ballot(e1 == e);
    const int before = __popcll(b0 & below) + __popcll(b1 & below);
    if (e0 == e) rank0 = before;
    if (e1 == e) rank1 = before;
    if (lane == 0) wave_cnt[wave][e] = __popcll(b0) + __popcll(b1);
  }
  __syncthreads();
  if (!live) return;
  int p0 = base[(int64_t)blockIdx.x * E + e0] + rank0;
  for (int w = 0; w < wave; ++w) p0 += wave_cnt[w][e0];
  slot_token[p0] = (int32_t)t;
  slot_scale[p0] = tw[2 * t];
  slot_dest[p0] = e1 >= 0 ? -1 : (int32_t)t;      // a skipped token's only slot (weight 1) is the token's output
  pos[2 * t] = p0;
  int p1 = -1;
  if (e1 >= 0) {
    p1 = base[(int64_t)blockIdx.x * E + e1] + rank1;
    for (int w = 0; w < wave; ++w) p1 += wave_cnt[w][e1];
    slot_token[p1] = (int32_t)t;
    slot_scale[p1] = tw[2 * t + 1];
    slot_dest[p1] = -1;
  }
  pos[2 * t + 1] = p1;
}

__device__ __forceinline__ uint32_t bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const float4* __restrict__ slot_out,
                                                      const int32_t* __restrict__ pos, int64_t T,
                                                      int H4, void* __restrict__ out, bool singles_done) {
  const int64_t n = T * H4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t t = i / H4;
    const int c = (int)(i - t * H4);
    const int p0 = pos[2 * t], p1 = pos[2 * t + 1];
    if (singles_done && p1 < 0) continue;       // written by the down projection
    float4 v = slot_out[(int64_t)p0 * H4 + c];
    if (p1 >= 0) {
      const float4 u = slot_out[(int64_t)p1 * H4 + c];
      v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
    }
    if (BF16) {
      uint2 o;
      o.x = bf16_rne(v.x) | (bf16_rne(v.y) << 16);
      o.y = bf16_rne(v.z) | (bf16_rne(v.w) << 16);
      ((uint2*)out)[i] = o;
    } else {
      ((float4*)out)[i] = v;
    }
  }
}


// ---- generalised top-k skipping -----------------------------------------------------------
template <int K>
__global__ __launch_bounds__(RB) void route_topk_kernel(const float* __restrict__ logits, int64_t T,
                                                        int E, uint32_t kept, double beta,
                                                        int32_t* __restrict__ n_used,
                                                        int32_t* __restrict__ topk,
                                                        float* __restrict__ tw,
                                                        int32_t* __restrict__ counts) {
  __shared__ int cnt[32];
  if (threadIdx.x < 32) cnt[threadIdx.x] = 0;
  __syncthreads();
  const int64_t t = (int64_t)blockIdx.x * RB + threadIdx.x;
  if (t < T) {
    const float* l = logits + t * E;
    uint32_t avail = kept;
    int es[K];
    double ex[K];
    float l_first = 0.f;
#pragma unroll
    for (int m = 0; m < K; ++m) {            // m-th largest kept logit; strict >: lower index wins a tie
      int best = -1;
      float bv = 0.f;
      for (int e = 0; e < E; ++e) {
        if (!((avail >> e) & 1u)) continue;
        const float v = l[e];
        if (best < 0 || v > bv) { best = e; bv = v; }
      }
      avail &= ~(1u << best);
      es[m] = best;
      if (m == 0) l_first = bv;
      ex[m] = exp((double)bv - (double)l_first);
    }
    double tail[K + 1];                      // tail[i] = sum_{m > i} w_m (m counted from 1)
    tail[K] = 0.0;
#pragma unroll
    for (int i = K - 1; i >= 0; --i) tail[i] = tail[i + 1] + ex[i];
    const double budget = beta * tail[0];
    int istar = K;
#pragma unroll
    for (int i = K - 1; i >= 1; --i)
      if (!(tail[i] > budget)) istar = i;    // ends at the smallest i that passes; tail[K] = 0 always passes
    // tails shrink with i, so "passes" is monotone and the smallest passing i is the answer
    double den = 0.0;
#pragma unroll
    for (int m = 0; m < K; ++m)
      if (m < istar) den += ex[m];
    n_used[t] = istar;
#pragma unroll
    for (int m = 0; m < K; ++m) {
      topk[t * K + m] = es[m];
      tw[t * K + m] = m < istar ? (float)(ex[m] / den) : 0.0f;
      if (m < istar) atomicAdd(&cnt[es[m]], 1);
    }
  }
  __syncthreads();
  if ((int)threadIdx.x < E) counts[(int64_t)blockIdx.x * E + threadIdx.x] = cnt[threadIdx.x];
}

template <int K>
__global__ __launch_bounds__(RB) void scatter_topk_kernel(const int32_t* __restrict__ topk,
                                                          const float* __restrict__ tw,
                                                          const int32_t* __restrict__ n_used,
                                                          const int32_t* __restrict__ base, int64_t T,
                                                          int E, int32_t* __restrict__ slot_token,
                                                          float* __restrict__ slot_scale,
                                                          int32_t* __restrict__ slot_dest,
                                                          int32_t* __restrict__ pos) {
  __shared__ int wave_cnt[RB / 64][32];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t t = (int64_t)blockIdx.x * RB + threadIdx.x;
  const bool live = t < T;
  const int nu = live ? n_used[t] : 0;
  int es[K], rank[K];
#pragma unroll
  for (int m = 0; m < K; ++m) { es[m] = m < nu ? topk[t * K + m] : -1; rank[m] = 0; }
  const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  for (int e = 0; e < E; ++e) {             // a token routes to an expert at most once
    bool has = false;
#pragma unroll
    for (int m = 0; m < K; ++m) has |= es[m] == e;
    const unsigned long long b = __ballot(has);
    const int before = __popcll(b & below);
#pragma unroll
    for (int m = 0; m < K; ++m)
      if (es[m] == e) rank[m] = before;
    if (lane == 0) wave_cnt[wave][e] = __popcll(b);
  }
  __syncthreads();
  if (!live) return;
#pragma unroll
  for (int m = 0; m < K; ++m) {
    int p = -1;
    if (es[m] >= 0) {
      p = base[(int64_t)blockIdx.x * E + es[m]] + rank[m];
      for (int w = 0; w < wave; ++w) p += wave_cnt[w][es[m]];
      slot_token[p] = (int32_t)t;
      slot_scale[p] = tw[t * K + m];
      slot_dest[p] = nu == 1 ? (int32_t)t : -1;     // a token's only slot (weight 1) is the token's output
    }
    pos[t * K + m] = p;
  }
}

template <bool BF16>
__global__ __launch_bounds__(256) void combine_topk_kernel(const float4* __restrict__ slot_out,
                                                           const int32_t* __restrict__ pos, int64_t T,
                                                           int H4, int K, void* __restrict__ out, bool singles_done) {
  const int64_t n = T * H4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t t = i / H4;
    const int c = (int)(i - t * H4);
    if (singles_done && (K == 1 || pos[t * K + 1] < 0)) continue;     // written by the down projection
    float4 v = slot_out[(int64_t)pos[t * K] * H4 + c];     // the best expert is always kept
    for (int m = 1; m < K; ++m) {
      const int p = pos[t * K + m];
      if (p < 0) break;                                   // kept experts are a prefix of the top-k
      const float4 u = slot_out[(int64_t)p * H4 + c];
      v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
    }
    if (BF16) {
      uint2 o;
      o.x = bf16_rne(v.x) | (bf16_rne(v.y) << 16);
      o.y = bf16_rne(v.z) | (bf16_rne(v.w) << 16);
      ((uint2*)out)[i] = o;
    } else {
      ((float4*)out)[i] = v;
    }
  }
}

}  // namespace

int plan_skip(int64_t T, int E, int H, int F, moep_dtype dt, int ks, SkipPlan* p, bool with_slot_out) {
  if ((int64_t)ks * T >= ((int64_t)1 << 31)) return fail(MOEP_EUNSUPPORTED, "moe_forward_skip: T too large");
  p->T = T; p->E = E; p->H = H; p->F = F; p->ks = ks;
  p->max_slots = (int64_t)ks * T;
  p->max_tiles = ceil_div((int64_t)ks * T, GEMM_BM) + E;
  const int64_t n_blocks = ceil_div(T, RB);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  p->off_logits = take((size_t)T * E * 4);
  p->off_slot_token = take((size_t)p->max_slots * 4);
  p->off_slot_scale = take((size_t)p->max_slots * 4);
  p->off_slot_dest = take((size_t)p->max_slots * 4);
  p->off_pos = take((size_t)T * ks * 4 * 3);           // pos, experts, weights: [T,ks] each
  p->off_counts = take((size_t)n_blocks * E * 4);
  p->off_seg_end = take((size_t)(2 * E + 1) * 4);          // segment ends, then each expert's first tile
  p->off_tile_expert = take((size_t)(p->max_tiles + 1) * 4);   // + the count of tiles in use
  p->off_tile_row0 = take((size_t)p->max_tiles * 4);
  p->packed = dt == MOEP_BF16;
  p->off_order_up = p->off_order_down = 0;
  if (dt == MOEP_BF16) {
    if (ceil_div(F, GEMM_BN_SWIGLU) > 4096 || ceil_div(H, GEMM_BN_STORE) > 4096 || p->max_tiles >= (1 << 20))
      return fail(MOEP_EUNSUPPORTED, "moe_forward_skip: too many tiles for the tile order tables");
    p->off_order_up = take((size_t)p->max_tiles * ceil_div(F, GEMM_BN_SWIGLU) * 4);
    p->off_order_down = take((size_t)p->max_tiles * ceil_div(H, GEMM_BN_STORE) * 4);
    // packed-operand GEMMs: h and the gathered x hold one 256-row block per tile; every expert's weights
    // are re-laid out once per call
    p->off_h = take(packed_a_bytes(p->max_tiles * GEMM_BM, F));
    p->off_xp = take(packed_a_bytes(p->max_tiles * GEMM_BM, H));
    p->off_w13 = take((size_t)E * packed_b_bytes(F, H, true));
    p->off_w2 = take((size_t)E * packed_b_bytes(H, F, false));
  } else {
    p->off_h = take((size_t)p->max_slots * F * dtype_size(dt));
    p->off_xp = p->off_w13 = p->off_w2 = 0;
  }
  p->off_slot_out = take(with_slot_out ? (size_t)p->max_slots * H * 4 : 0);
  p->total = off > 0 ? off : 256;
  return MOEP_OK;
}

// Tile order tables of the two grouped projections (bf16 path), from the tile map scan_kernel has just written.
static void launch_order_tables(const SkipPlan& p, char* ws, hipStream_t s) {
  if (!p.packed) return;
  const int32_t* expert_first = (const int32_t*)(ws + p.off_seg_end) + p.E;
  const int n_up = (int)ceil_div(p.F, GEMM_BN_SWIGLU), n_down = (int)ceil_div(p.H, GEMM_BN_STORE);
  hipLaunchKernelGGL(order_kernel, dim3((unsigned)ceil_div(p.max_tiles * n_up, 256)), dim3(256), 0, s, expert_first, p.E,
                     n_up, GEMM_GROUP_M_SWIGLU, (uint32_t*)(ws + p.off_order_up));
  hipLaunchKernelGGL(order_kernel, dim3((unsigned)ceil_div(p.max_tiles * n_down, 256)), dim3(256), 0, s, expert_first, p.E,
                     n_down, GEMM_GROUP_M_STORE, (uint32_t*)(ws + p.off_order_down));
}

int launch_skip_routing(const SkipPlan& p, const float* logits, uint32_t kept_mask, float beta, uint8_t* skip_mask,
                        int32_t* top2_out, char* ws, hipStream_t s) {
  const int64_t T = p.T;
  int32_t* pos = (int32_t*)(ws + p.off_pos);
  int32_t* top2 = top2_out ? top2_out : pos + 2 * T;
  float* tw = (float*)(pos + 4 * T);
  int32_t* counts = (int32_t*)(ws + p.off_counts);
  const int64_t n_blocks = ceil_div(T, RB);
  const float theta = beta > 0.0f ? (float)std::log((double)beta) : -INFINITY;
  Timed t("skip_route_dispatch", s);
  hipLaunchKernelGGL(route_kernel, dim3((unsigned)n_blocks), dim3(RB), 0, s, logits, T, p.E, kept_mask, theta,
                     skip_mask, top2, tw, counts);
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(256), 0, s, counts, n_blocks, p.E,
                     (int32_t*)(ws + p.off_seg_end), (int32_t*)(ws + p.off_tile_expert),
                     (int32_t*)(ws + p.off_tile_row0), (int)p.max_tiles);
  launch_order_tables(p, ws, s);
  hipLaunchKernelGGL(scatter_kernel, dim3((unsigned)n_blocks), dim3(RB), 0, s, top2, tw, skip_mask,
                     counts, T, p.E, (int32_t*)(ws + p.off_slot_token),
                     (float*)(ws + p.off_slot_scale), (int32_t*)(ws + p.off_slot_dest), pos);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

int launch_skip_combine(const SkipPlan& p, moep_dtype dt, const uint8_t* skip_mask, void* out,
                        char* ws, hipStream_t s, bool singles_done) {
  (void)skip_mask;
  const int H4 = p.H / 4;
  const int64_t n = p.T * H4;
  const unsigned blocks = (unsigned)(ceil_div(n, 256) < 65536 ? ceil_div(n, 256) : 65536);
  Timed t("skip_combine", s);
  if (dt == MOEP_BF16)
    hipLaunchKernelGGL(combine_kernel<true>, dim3(blocks), dim3(256), 0, s,
                       (const float4*)(ws + p.off_slot_out), (const int32_t*)(ws + p.off_pos), p.T, H4, out, singles_done);
  else
    hipLaunchKernelGGL(combine_kernel<false>, dim3(blocks), dim3(256), 0, s,
                       (const float4*)(ws + p.off_slot_out), (const int32_t*)(ws + p.off_pos), p.T, H4, out, singles_done);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}


int launch_skip_topk_routing(const SkipPlan& p, const float* logits, uint32_t kept_mask, float beta,
                             int32_t* n_used, int32_t* topk_out, char* ws, hipStream_t s, int32_t* pos_out) {
  const int64_t T = p.T;
  const int K = p.ks;
  int32_t* ws_pos = (int32_t*)(ws + p.off_pos);
  int32_t* pos = pos_out ? pos_out : ws_pos;
  int32_t* topk = topk_out ? topk_out : ws_pos + (int64_t)K * T;
  float* tw = (float*)(ws_pos + 2 * (int64_t)K * T);
  int32_t* counts = (int32_t*)(ws + p.off_counts);
  const int64_t n_blocks = ceil_div(T, RB);
  int32_t* slot_token = (int32_t*)(ws + p.off_slot_token);
  float* slot_scale = (float*)(ws + p.off_slot_scale);
  int32_t* slot_dest = (int32_t*)(ws + p.off_slot_dest);
  Timed t("skip_route_dispatch", s);
#define MOEP_ROUTE_CASE(KK)                                                                    \
  case KK:                                                                                    \
    hipLaunchKernelGGL(route_topk_kernel<KK>, dim3((unsigned)n_blocks), dim3(RB), 0, s, logits, T, p.E, \
                       kept_mask, (double)beta, n_used, topk, tw, counts);                    \
    break;
  switch (K) {
    MOEP_ROUTE_CASE(1) MOEP_ROUTE_CASE(2) MOEP_ROUTE_CASE(3) MOEP_ROUTE_CASE(4)
    MOEP_ROUTE_CASE(5) MOEP_ROUTE_CASE(6) MOEP_ROUTE_CASE(7) MOEP_ROUTE_CASE(8)
    MOEP_ROUTE_CASE(9) MOEP_ROUTE_CASE(10) MOEP_ROUTE_CASE(11) MOEP_ROUTE_CASE(12)
    MOEP_ROUTE_CASE(13) MOEP_ROUTE_CASE(14) MOEP_ROUTE_CASE(15) MOEP_ROUTE_CASE(16)
    default: return fail(MOEP_EUNSUPPORTED, "top-k routing: k=%d (1..16)", K);
  }
#undef MOEP_ROUTE_CASE
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(256), 0, s, counts, n_blocks, p.E,
                     (int32_t*)(ws + p.off_seg_end), (int32_t*)(ws + p.off_tile_expert),
                     (int32_t*)(ws + p.off_tile_row0), (int)p.max_tiles);
  launch_order_tables(p, ws, s);
#define MOEP_SCATTER_CASE(KK)                                                                  \
  case KK:                                                                                    \
    hipLaunchKernelGGL(scatter_topk_kernel<KK>, dim3((unsigned)n_blocks), dim3(RB), 0, s, topk, tw, \
                       n_used, counts, T, p.E, slot_token, slot_scale, slot_dest, pos);       \
    break;
  switch (K) {
    MOEP_SCATTER_CASE(1) MOEP_SCATTER_CASE(2) MOEP_SCATTER_CASE(3) MOEP_SCATTER_CASE(4)
    MOEP_SCATTER_CASE(5) MOEP_SCATTER_CASE(6) MOEP_SCATTER_CASE(7) MOEP_SCATTER_CASE(8)
    MOEP_SCATTER_CASE(9) MOEP_SCATTER_CASE(10) MOEP_SCATTER_CASE(11) MOEP_SCATTER_CASE(12)
    MOEP_SCATTER_CASE(13) MOEP_SCATTER_CASE(14) MOEP_SCATTER_CASE(15) MOEP_SCATTER_CASE(16)
  }
#undef MOEP_SCATTER_CASE
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

int launch_skip_topk_combine(const SkipPlan& p, moep_dtype dt, void* out, char* ws, hipStream_t s, bool singles_done) {
  const int H4 = p.H / 4;
  const int64_t n = p.T * H4;
  const unsigned blocks = (unsigned)(ceil_div(n, 256) < 65536 ? ceil_div(n, 256) : 65536);
  Timed t("skip_combine", s);
  if (dt == MOEP_BF16)
    hipLaunchKernelGGL(combine_topk_kernel<true>, dim3(blocks), dim3(256), 0, s,
                       (const float4*)(ws + p.off_slot_out), (const int32_t*)(ws + p.off_pos), p.T, H4, p.ks, out, singles_done);
  else
    hipLaunchKernelGGL(combine_topk_kernel<false>, dim3(blocks), dim3(256), 0, s,
                       (const float4*)(ws + p.off_slot_out), (const int32_t*)(ws + p.off_pos), p.T, H4, p.ks, out, singles_done);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

}  // namespace moep
