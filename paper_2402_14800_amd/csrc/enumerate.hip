// Enumeration of kept-expert subsets (Sec. 3.2, Eq. 3) through the per-token Gram matrix.
//
// For token t let Y_t be the E x H matrix of its expert outputs, a the Eq. 1 weights of the full
// layer (top-k of all experts) and b those of the layer pruned to the kept set C (top-min(k,r)
// of C).  Then F'(x_t,C) - F(x_t) = sum_e (b_e - a_e) Y_t[e,:] and its squared norm is d^T G_t d
// with d = b - a, G_t = Y_t Y_t^T.  The kernels:
//
//   gram        G_t for every token: the only pass over Y (HBM-bound).  bf16: rows are fetched in whole
//               1 KB pieces, turned into MFMA fragments through wave-private LDS, and multiplied with
//               one v_mfma_f32_16x16x32_bf16 per 16 rows x 32 hidden units, the SAME registers feeding
//               both operands (B = A^T); two tokens per tile when E <= 8.
//   prep        per token: stable descending order of the logits (ties -> lower index), and
//               everything the scorer needs, moved to RANK space (position j = j-th ranked expert):
//               exp(l_j - l_0), l_j, the full-layer weights a_j, the Gram matrix permuted to rank
//               order (off-diagonals doubled).  Only the first n_act = min(E, min(k,r) + E - r)
//               positions can ever be selected by a pruned layer, so only those are kept.
//   score       lane = subset, loop over a tile of tokens.  Per token all data is wave-uniform
//               (scalar loads); each lane walks the rank positions, takes the first min(k,r) whose
//               expert is in its mask, forms d explicitly and evaluates d^T G d.  A pair whose
//               selection equals the full top-k contributes exactly 0 and is counted.
//   score (many subsets)  A token's error depends on the subset only through WHICH of its first n_act ranked experts
//               are kept, and then only through the first min(k,r) of those: C(n_act, min(k,r)) possible selections per
//               token against C(E,r) subsets (495 against 12870 for E = 16, k = 4, r = 8).  qtable evaluates the error
//               of every selection once per token; score_lut then needs, per (subset, token), a few table look-ups:
//               kept mask -> pattern of kept rank positions (nibble tables built per token from its order),
//               pattern -> selection index (one table per launch), selection index -> error.
//   reduce      loss[i] = sum over token tiles of the partial sums, in a fixed order (fp64 adds).
//   argmin      lowest index attaining the minimum; its mask by lexicographic unranking.
#include "common.h"

namespace moep {
namespace {

// ------------------------------------------------------------------ binomials / unranking
struct BinomTable {
  uint32_t v[33][33];
  constexpr BinomTable() : v{} {
    for (int n = 0; n <= 32; ++n) {
      v[n][0] = 1;
      for (int r = 1; r <= n; ++r) v[n][r] = v[n - 1][r - 1] + (r <= n - 1 ? v[n - 1][r] : 0);
    }
  }
};
__constant__ BinomTable c_binom = BinomTable();

// Kept mask of subset `idx` in lexicographic order of sorted r-tuples over {0..E-1}.
__device__ uint32_t unrank_device(int E, int r, uint32_t idx) {
  uint32_t mask = 0;
  int rem = r;
  for (int e = 0; e < E; ++e) {
    if (rem == 0) break;
    const uint32_t with_e = c_binom.v[E - 1 - e][rem - 1];
    if (idx < with_e) { mask |= 1u << e; --rem; }
    else idx -= with_e;
  }
  return mask;
}

__global__ __launch_bounds__(256) void masks_kernel(int E, int r, uint32_t n_sub, uint32_t* __restrict__ masks) {
  const uint32_t i = blockIdx.x * 256 + threadIdx.x;
  if (i < n_sub) masks[i] = unrank_device(E, r, i);
}

// ------------------------------------------------------------------ Gram, bf16 (MFMA)
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// EPAD = rows reserved per token inside a 16-row MFMA tile (4, 8 or 16): 16 / EPAD tokens per tile, one
// tile per wavefront; the 8x8 (4x4) blocks of the 16x16 product that pair different tokens are discarded.
// RANKED: the rows are the outputs of each token's n best-ranked experts, addressed through
// slot_of[t, j], with experts[t, j] naming the expert; G keeps its expert indexing (see below).
//
// A wavefront fetches each of the tile's 16 rows in whole 1 KB pieces (64 lanes x 16 bytes of ONE row per
// load), so that a DRAM page is read in one go wherever the 16 rows lie: with E T H a power of two the
// expert rows of a token fall into the same DRAM bank, and fragment-shaped loads (64 bytes of each of
// 16 rows per instruction) keep re-opening 16 pages of that bank (measured 4.8 against 5.7 TB/s at E = 16).
// The pieces become MFMA fragments through a wave-private 16 KB of LDS (chunk c of row j at position
// c ^ j: the row-wise writes and the column-wise fragment reads are both free of bank conflicts); the next
// 16 loads are in flight in registers while the current block of 512 hidden units is multiplied.  The
// same registers serve as both MFMA operands (B = A^T).
// STREAM: Y is far larger than the caches, so its loads carry the non-temporal hint (measured 6.2 -> 6.8 TB/s at
// 17 GB and 5.6 -> 6.0 TB/s at 4.3 GB; a Y of a few hundred MB that the down projection has just written is
// better read with ordinary loads: 6.5 against 5.0 TB/s at 0.27 GB).
// 16 bytes of Y with the non-temporal hint: a stream read once, not worth a place in the caches.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_streaming(const uint4* p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v[0], v[1], v[2], v[3]);
}

template <int EPAD, bool RANKED, bool STREAM>
__global__ __launch_bounds__(256) void gram_bf16_kernel(const uint4* __restrict__ Y,
                                                        const int32_t* __restrict__ slot_of,
                                                        const int32_t* __restrict__ experts,
                                                        float* __restrict__ G, int64_t T, int E, int n,
                                                        int H) {
  constexpr int TPT = 16 / EPAD;
  __shared__ uint4 stage[4][16 * 64];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
  const int64_t t0 = tile * TPT;
  if (t0 >= T) return;
  uint4* st = stage[wave];
  const int chunks = H / 8;                             // 16-byte chunks per row
  const int nkb = (chunks + 63) / 64;                   // blocks of 512 hidden units
  // row j of the tile: expert (rank position) j % EPAD of token t0 + j / EPAD; rows without data read as zeros
  const uint4* rowp[16];
  bool rvalid[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int e = j % EPAD;
    const int64_t t = t0 + j / EPAD;
    rvalid[j] = e < (RANKED ? n : E) && t < T;
    int64_t r = 0;
    if (rvalid[j]) r = RANKED ? (int64_t)slot_of[t * n + e] : (int64_t)e * T + t;
    rowp[j] = Y + r * chunks + lane;
  }
  const int row = lane & 15, kg = lane >> 4;
  f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = acc0;
  uint4 v[16];
#define MOEP_GRAM_FETCH(kb)                                                                     \
  _Pragma("unroll") for (int j = 0; j < 16; ++j)                                                \
    v[j] = !(rvalid[j] && (kb) * 64 + lane < chunks) ? make_uint4(0, 0, 0, 0)                    \
           : STREAM ? load_streaming(&rowp[j][(kb) * 64]) : rowp[j][(kb) * 64];
  MOEP_GRAM_FETCH(0)
  for (int kb = 0; kb < nkb; ++kb) {
#pragma unroll
    for (int j = 0; j < 16; ++j) st[j * 64 + (lane ^ j)] = v[j];
    if (kb + 1 < nkb) { MOEP_GRAM_FETCH(kb + 1) }
    // MFMA 16x16x32: lane l supplies row (l & 15) and 8 consecutive hidden units; which 8 is free as long as
    // every row agrees, here chunk 4 s + (l >> 4) of the block
#pragma unroll
    for (int s = 0; s < 16; s += 2) {
      const bf16x8 a0 = __builtin_bit_cast(bf16x8, st[row * 64 + ((4 * s + kg) ^ row)]);
      const bf16x8 a1 = __builtin_bit_cast(bf16x8, st[row * 64 + ((4 * (s + 1) + kg) ^ row)]);
      acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, a0, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, a1, acc1, 0, 0, 0);
    }
  }
#undef MOEP_GRAM_FETCH
  // Accumulator layout of the 16x16 tile: register v of lane l = row 4 (l / 16) + v, column l % 16.
  const int col = lane & 15;
  const int cj = col % EPAD;
  const int64_t ct = t0 + col / EPAD;
  if (ct >= T || cj >= (RANKED ? n : E)) return;
  const int ce = RANKED ? experts[ct * n + cj] : cj;
#pragma unroll
  for (int vv = 0; vv < 4; ++vv) {
    const int r = 4 * (lane >> 4) + vv;
    const int rj = r % EPAD;
    if (r / EPAD == col / EPAD && rj < (RANKED ? n : E)) {
      const int re = RANKED ? experts[ct * n + rj] : rj;
      G[(ct * E + re) * E + ce] = acc0[vv] + acc1[vv];
    }
  }
}

// E in 17..32: one token per 32x32 tile.
__global__ __launch_bounds__(256) void gram_bf16_32_kernel(const uint4* __restrict__ Y,
                                                           float* __restrict__ G, int64_t T, int E,
                                                           int H) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const int row = lane & 31, kg = lane >> 5;
  const bool valid = row < E;
  const int chunks = H / 8;
  const uint4* src = Y + ((int64_t)(valid ? row : 0) * T + t) * chunks + kg;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  const int steps = H / 16;
  for (int s0 = 0; s0 < steps; s0 += 4) {
    uint4 v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = valid ? src[(s0 + i) * 2] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, v[i]);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, a, acc, 0, 0, 0);
    }
  }
  const int col = lane & 31;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int r = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    if (r < E && col < E) G[(t * E + r) * E + col] = acc[v];
  }
}

// ------------------------------------------------------------------ Gram, fp32 storage
__global__ __launch_bounds__(256) void gram_f32_kernel(const float* __restrict__ Y,
                                                       float* __restrict__ G, int64_t T, int E,
                                                       int H) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  for (int e = 0; e < E; ++e)
    for (int f = e; f < E; ++f) {
      const float* ye = Y + ((int64_t)e * T + t) * H;
      const float* yf = Y + ((int64_t)f * T + t) * H;
      float s = 0.f;
      for (int h = lane; h < H; h += 64) s = fmaf(ye[h], yf[h], s);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
      if (lane == 0) {
        G[(t * E + e) * E + f] = s;
        G[(t * E + f) * E + e] = s;
      }
    }
}


// ------------------------------------------------------------------ Gram from ranked expert outputs
// The rank-limited expert pass stores, per token, only the outputs of its n best-ranked experts, as
// rows of Yr addressed through slot_of[t, j]; experts[t, j] names the expert.  G keeps its expert
// indexing: entry (e_i, e_j) of token t is written for the token's n ranked experts only, which is
// every entry the routing-prep kernel reads as long as n >= n_act.
__global__ __launch_bounds__(256) void gram_ranked_f32_kernel(const float* __restrict__ Yr,
                                                              const int32_t* __restrict__ slot_of,
                                                              const int32_t* __restrict__ experts,
                                                              float* __restrict__ G, int64_t T, int E,
                                                              int n, int H) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  for (int i = 0; i < n; ++i)
    for (int j = i; j < n; ++j) {
      const float* yi = Yr + (int64_t)slot_of[t * n + i] * H;
      const float* yj = Yr + (int64_t)slot_of[t * n + j] * H;
      float s = 0.f;
      for (int h = lane; h < H; h += 64) s = fmaf(yi[h], yj[h], s);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
      if (lane == 0) {
        const int ei = experts[t * n + i], ej = experts[t * n + j];
        G[(t * E + ei) * E + ej] = s;
        G[(t * E + ej) * E + ei] = s;
      }
    }
}

// ------------------------------------------------------------------ record layout
// Per token, CAP = capacity >= n_act, all fp32 unless noted:
//   [0, CAP)            ex_j  = exp(l_j - l_0), l in rank order (0 beyond n_act)
//   [CAP, 2 CAP)        l_j
//   [2 CAP, 3 CAP)      a_j   = full-layer Eq. 1 weight of rank j (0 for j >= k)
//   [3 CAP, 3 CAP + CAP (CAP + 1) / 2)   Gram in rank order, row-major upper triangle,
//                       diagonal as is, off-diagonal entries doubled
//   then ceil(CAP / 4) words: expert index of rank j in byte j
__host__ __device__ constexpr int rec_tri(int cap) { return cap * (cap + 1) / 2; }
__host__ __device__ constexpr int rec_order_off(int cap) { return 3 * cap + rec_tri(cap); }
__host__ __device__ constexpr int rec_size(int cap) {
  return (rec_order_off(cap) + (cap + 3) / 4 + 3) & ~3;
}

// One thread per token.  STAGED: the thread builds its record in LDS (rec_floats + 1 words apart: no bank conflicts)
// and the workgroup then writes its tokens' records, which are consecutive in memory, in 16-byte pieces; otherwise
// (records too large for the LDS) every thread writes its own record word by word.
template <int EMAX, bool STAGED>
__global__ __launch_bounds__(256) void prep_kernel(const float* __restrict__ logits,
                                                   const float* __restrict__ G,
                                                   float* __restrict__ rec, int64_t T, int E,
                                                   int k, int n_act, int cap, int rec_floats) {
  extern __shared__ float stage[];
  const int64_t t0 = (int64_t)blockIdx.x * blockDim.x;
  const int64_t t = t0 + threadIdx.x;
  if (t < T) {
  float l[EMAX];
#pragma unroll
  for (int e = 0; e < EMAX; ++e) l[e] = e < E ? logits[t * E + e] : 0.f;
  // rank of expert e = number of experts that precede it: larger logit, or equal and lower index
  int rank[EMAX];
#pragma unroll
  for (int e = 0; e < EMAX; ++e) {
    int c = 0;
#pragma unroll
    for (int f = 0; f < EMAX; ++f)
      if (f < E && f != e) c += (l[f] > l[e] || (l[f] == l[e] && f < e)) ? 1 : 0;
    rank[e] = e < E ? c : 255;
  }
  float* R = STAGED ? stage + threadIdx.x * (rec_floats + 1) : rec + t * rec_floats;
  for (int i = 0; i < rec_floats; ++i) R[i] = 0.f;
  uint32_t* Rord = (uint32_t*)(R + rec_order_off(cap));
  int ord[EMAX];
  float l0 = 0.f;
  for (int j = 0; j < n_act; ++j) {
    int oe = 0;
    float lv = 0.f;
#pragma unroll
    for (int e = 0; e < EMAX; ++e)
      if (rank[e] == j) { oe = e; lv = l[e]; }
    ord[j] = oe;
    if (j == 0) l0 = lv;
    R[j] = expf(lv - l0);
    R[cap + j] = lv;
  }
  float den = 0.f;
  for (int j = 0; j < k; ++j) den += R[j];
  for (int j = 0; j < k; ++j) R[2 * cap + j] = R[j] / den;
  int idx = 3 * cap;
  for (int i = 0; i < cap; ++i)
    for (int j = i; j < cap; ++j, ++idx)
      if (i < n_act && j < n_act) {
        const float g = G[(t * E + ord[i]) * E + ord[j]];
        R[idx] = i == j ? g : 2.0f * g;
      }
  for (int w = 0; w < (cap + 3) / 4; ++w) {
    uint32_t packed = 0;
    for (int b = 0; b < 4; ++b) {
      const int j = 4 * w + b;
      if (j < n_act) packed |= (uint32_t)ord[j] << (8 * b);
    }
    Rord[w] = packed;
  }
  }
  if (STAGED) {
    __syncthreads();
    const int64_t left = T - t0;
    const int words = (int)(left < (int64_t)blockDim.x ? left : (int64_t)blockDim.x) * rec_floats;   // a multiple of 4
    float4* dst = (float4*)(rec + t0 * rec_floats);
    for (int q = 4 * threadIdx.x; q < words; q += 4 * blockDim.x) {
      const float* src = stage + (q / rec_floats) * (rec_floats + 1) + q % rec_floats;   // the 4 words are one token's
      dst[q >> 2] = make_float4(src[0], src[1], src[2], src[3]);
    }
  }
}

// ------------------------------------------------------------------ scoring
// EXACT: every one of the CAP rank positions is in use (n_act == CAP), which removes the
// per-position guards from the token loop.
template <int CAP, bool EXACT>
__global__ __launch_bounds__(256) void score_kernel(const float* __restrict__ rec, int64_t T,
                                                    int tok_tile, int E, int r, int kk, int kfull,
                                                    int n_act_rt, uint32_t n_sub,
                                                    float* __restrict__ partial,
                                                    uint32_t* __restrict__ partial_cnt) {
  constexpr int RS = rec_size(CAP);
  const int n_act = EXACT ? CAP : n_act_rt;
  constexpr int OFF_L = CAP, OFF_A = 2 * CAP, OFF_G = 3 * CAP, OFF_O = rec_order_off(CAP);
  const uint32_t sub = blockIdx.x * blockDim.x + threadIdx.x;
  const bool live = sub < n_sub;
  // Idle lanes keep every expert: their selection always equals the full one and costs nothing.
  const uint32_t mask = live ? unrank_device(E, r, sub) : 0xffffffffu;
  const uint32_t full_bits = kk != kfull ? 0u : (kfull >= 32 ? 0xffffffffu : (1u << kfull) - 1u);   // r < k: never "same"
  const int64_t t_begin = (int64_t)blockIdx.y * tok_tile;
  const int64_t t_end = t_begin + tok_tile < T ? t_begin + tok_tile : T;

  float total = 0.f;
  uint32_t same_cnt = 0;
  for (int64_t t = t_begin; t < t_end; ++t) {
    const float* R = rec + t * RS;                       // wave-uniform
    const uint32_t* Rord = (const uint32_t*)(R + OFF_O);
    // Everything the selection needs is fetched up front, unconditionally (wave-uniform scalar
    // loads), so that no load sits behind a lane-dependent condition.
    float ex[CAP], aw[CAP];
    uint32_t ordw[(CAP + 3) / 4];
#pragma unroll
    for (int j = 0; j < CAP; ++j) { ex[j] = R[j]; aw[j] = R[OFF_A + j]; }
#pragma unroll
    for (int j = 0; j < (CAP + 3) / 4; ++j) ordw[j] = Rord[j];
    float w[CAP];
    float sum = 0.f;
    uint32_t bits = 0;
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < CAP; ++j) {
      w[j] = 0.f;
      if (j < n_act) {
        const uint32_t e = (ordw[j >> 2] >> (8 * (j & 3))) & 0xffu;
        const bool take = ((mask >> e) & 1u) && cnt < kk;
        cnt += take ? 1 : 0;
        bits |= take ? (1u << j) : 0u;
        w[j] = take ? ex[j] : 0.f;
        sum += w[j];
      }
    }
    if (sum < 1e-30f) {
      // Every selected logit lies far below the token's maximum: redo Eq. 1 relative to the
      // largest SELECTED logit (the first one taken), as the definition has it.
      float m = 0.f;
      bool have = false;
#pragma unroll
      for (int j = 0; j < CAP; ++j)
        if (j < n_act && ((bits >> j) & 1u) && !have) { m = R[OFF_L + j]; have = true; }
      sum = 0.f;
#pragma unroll
      for (int j = 0; j < CAP; ++j) {
        w[j] = (j < n_act && ((bits >> j) & 1u)) ? __expf(R[OFF_L + j] - m) : 0.f;
        sum += w[j];
      }
    }
    const float inv = __builtin_amdgcn_rcpf(sum);
    float d[CAP];
#pragma unroll
    for (int j = 0; j < CAP; ++j) d[j] = fmaf(w[j], inv, -aw[j]);
    float q = 0.f;
    int gi = OFF_G;
#pragma unroll
    for (int i = 0; i < CAP; ++i) {
      float u = 0.f;
#pragma unroll
      for (int j = i; j < CAP; ++j, ++gi) u = fmaf(R[gi], d[j], u);
      q = fmaf(d[i], u, q);
    }
    const bool same = bits == full_bits;
    same_cnt += (same && live) ? 1u : 0u;
    total += same ? 0.f : q;
  }
  if (live) {
    partial[(int64_t)blockIdx.y * n_sub + sub] = total;
    partial_cnt[(int64_t)blockIdx.y * n_sub + sub] = same_cnt;
  }
}

// ------------------------------------------------------------------ scoring through per-token selection tables
// Rank of the selection made by the kept-position pattern `pat` (bit j = the token's j-th ranked expert is kept):
// the first kk set bits, as a kk-subset of the n_act positions, indexed in lexicographic order (index 0 = positions
// 0 .. kk-1 = the selection of the full layer when kk = k).  Patterns with fewer than kk bits belong to no subset.
// selbits[i] = the positions of selection i (the pattern with exactly kk bits that has index i).
__global__ __launch_bounds__(256) void selidx_kernel(int n_act, int kk, uint16_t* __restrict__ sel,
                                                     uint16_t* __restrict__ selbits) {
  const uint32_t pat = blockIdx.x * 256 + threadIdx.x;
  if (pat >= (1u << n_act)) return;
  uint32_t idx = 0;
  int rem = kk;
  for (int j = 0; j < n_act && rem > 0; ++j) {
    if ((pat >> j) & 1u) --rem;
    else idx += c_binom.v[n_act - 1 - j][rem - 1];     // all selections whose next position is j come first
  }
  sel[pat] = rem == 0 ? (uint16_t)idx : (uint16_t)1;     // too few bits: only idle lanes look these up (never index 0)
  if (rem == 0 && __popc(pat) == kk) selbits[idx] = (uint16_t)pat;
}

// One workgroup per token: the error d^T G d of every selection (kk of the first n_act rank positions), the same
// arithmetic as score_kernel's.  Selection 0 is the full layer's when kk = kfull: exactly 0.
template <int CAP, bool EXACT>
__global__ __launch_bounds__(256) void qtable_kernel(const float* __restrict__ rec, int kk, int kfull, int n_act_rt,
                                                     int n_combo, const uint16_t* __restrict__ selbits,
                                                     float* __restrict__ qtab, int nib,
                                                     uint16_t* __restrict__ nibtab) {
  constexpr int RS = rec_size(CAP);
  const int n_act = EXACT ? CAP : n_act_rt;
  constexpr int OFF_L = CAP, OFF_A = 2 * CAP, OFF_G = 3 * CAP;
  const int64_t t = blockIdx.x;
  const float* R = rec + t * RS;                        // wave-uniform
  float ex[CAP], aw[CAP];
#pragma unroll
  for (int j = 0; j < CAP; ++j) { ex[j] = R[j]; aw[j] = R[OFF_A + j]; }
  for (int c = threadIdx.x; c < n_combo; c += blockDim.x) {
    const uint32_t bits = selbits[c];
    float w[CAP];
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < CAP; ++j) {
      w[j] = (j < n_act && ((bits >> j) & 1u)) ? ex[j] : 0.f;
      sum += w[j];
    }
    if (sum < 1e-30f) {                                  // see score_kernel
      float m = 0.f;
      bool have = false;
#pragma unroll
      for (int j = 0; j < CAP; ++j)
        if (j < n_act && ((bits >> j) & 1u) && !have) { m = R[OFF_L + j]; have = true; }
      sum = 0.f;
#pragma unroll
      for (int j = 0; j < CAP; ++j) {
        w[j] = (j < n_act && ((bits >> j) & 1u)) ? __expf(R[OFF_L + j] - m) : 0.f;
        sum += w[j];
      }
    }
    const float inv = __builtin_amdgcn_rcpf(sum);
    float d[CAP];
#pragma unroll
    for (int j = 0; j < CAP; ++j) d[j] = fmaf(w[j], inv, -aw[j]);
    float q = 0.f;
    int gi = OFF_G;
#pragma unroll
    for (int i = 0; i < CAP; ++i) {
      float u = 0.f;
#pragma unroll
      for (int j = i; j < CAP; ++j, ++gi) u = fmaf(R[gi], d[j], u);
      q = fmaf(d[i], u, q);
    }
    qtab[t * n_combo + c] = (c == 0 && kk == kfull) ? 0.f : q;
  }
  // The token's nibble tables, which turn a kept mask into a kept-position pattern four experts at a time: entry v
  // of nibble nb = the rank positions (below n_act) of the experts 4 nb + b with bit b of v set.  Stored as the low
  // or high half of a 32-bit word shared with the neighbouring token, so that one look-up serves two tokens.
  const uint32_t* ordw = (const uint32_t*)(R + rec_order_off(CAP));
  for (int q = threadIdx.x; q < nib * 16; q += blockDim.x) {
    const int nb = q >> 4, v = q & 15;
    uint32_t pat = 0;
    for (int j = 0; j < n_act; ++j) {
      const uint32_t e = (ordw[j >> 2] >> (8 * (j & 3))) & 0xffu;
      if ((int)(e >> 2) == nb && ((v >> (e & 3)) & 1)) pat |= 1u << j;
    }
    nibtab[((t >> 1) * (nib * 16) + q) * 2 + (t & 1)] = (uint16_t)pat;   // tokens 2 i and 2 i + 1 share a word
  }
}

// Lane = SPL subsets, loop over a tile of tokens, LUT_TG tokens per barrier (double-buffered in LDS).  Per pair:
// one look-up per nibble of the kept mask (lanes of a wavefront hold neighbouring subsets: few distinct entries, no
// bank conflicts), one of the pattern's selection index, one of that selection's error.
constexpr int LUT_TG = 8, LUT_MAX_ACT = 12, LUT_MAX_COMBO = 512, LUT_MAX_ADDR = 68;
// Where the pattern table keeps pattern `pat` in LDS: pattern bits 6..10 folded onto the bits that choose the bank.
// The patterns of a wavefront's 64 subsets differ in the few rank positions of the experts that vary among them, any
// of the n_act; left to bits 1..5 alone the bank would ignore the rest and they would queue on a few banks.
__device__ __forceinline__ uint32_t lut_swizzle(uint32_t pat) { return pat ^ ((pat >> 5) & 0x3eu); }

template <int NIB, int SPL>    // NIB = nibbles of the kept mask: ceil(E / 4)
__global__ __launch_bounds__(256, 3) void score_lut_kernel(const float* __restrict__ qtab,
                                                        const uint32_t* __restrict__ nibtab,
                                                        const uint16_t* __restrict__ sel, int64_t T, int tok_tile,
                                                        int E, int r, int n_act, int n_combo, bool count_same,
                                                        uint32_t n_sub, float* __restrict__ partial,
                                                        uint32_t* __restrict__ partial_cnt) {
  constexpr int NT = NIB * 16;                           // nibble-table entries per token
  __shared__ uint16_t s_sel[1 << LUT_MAX_ACT];
  __shared__ uint32_t s_nib[2][LUT_TG / 2 * NT];
  __shared__ float s_q[2][LUT_TG * LUT_MAX_COMBO];
  const int tid = threadIdx.x;
  for (int i = tid; i < (1 << n_act); i += 256) s_sel[lut_swizzle((uint32_t)i)] = sel[i];
  uint32_t mask[SPL];
  float total[SPL];
  uint32_t same_cnt = 0;                                 // over all of the lane's subsets
#pragma unroll
  for (int s = 0; s < SPL; ++s) {
    const uint32_t sub = (blockIdx.x * SPL + s) * 256 + tid;
    mask[s] = sub < n_sub ? unrank_device(E, r, sub) : 0u;   // idle: empty pattern, selection index 1, not counted
    total[s] = 0.f;
  }
  const int64_t t_begin = (int64_t)blockIdx.y * tok_tile;
  const int64_t t_end = t_begin + tok_tile < T ? t_begin + tok_tile : T;
  int buf = 0;
  for (int64_t g0 = t_begin; g0 < t_end; g0 += LUT_TG, buf ^= 1) {
    const int ntok = (int)(t_end - g0 < LUT_TG ? t_end - g0 : LUT_TG);
    {
      const uint32_t* src = nibtab + (g0 >> 1) * NT;       // g0 is even
      for (int i = tid; i < ((ntok + 1) >> 1) * NT; i += 256) s_nib[buf][i] = src[i];
    }
    // the group's selection errors: ntok x n_combo consecutive floats
    {
      const float* src = qtab + g0 * n_combo;
      for (int i = tid; i < ntok * n_combo; i += 256) s_q[buf][i] = src[i];
    }
    __syncthreads();      // (also covers s_sel on the first pass; the other buffer is still being read by nobody:
                          //  every thread finished its look-ups in it before it arrived at the previous barrier)
    for (int tk = 0; tk < ntok; tk += 2) {
      const uint32_t* nib = s_nib[buf] + (tk >> 1) * NT;
      const float* qrow = s_q[buf] + tk * n_combo;
      const bool pair = tk + 1 < ntok;                   // the group's last token may stand alone
#pragma unroll
      for (int s = 0; s < SPL; ++s) {
        uint32_t pat = 0;                                // low half: token tk, high half: token tk + 1
#pragma unroll
        for (int nb = 0; nb < NIB; ++nb) pat |= nib[nb * 16 + ((mask[s] >> (4 * nb)) & 15u)];
        const uint32_t si0 = s_sel[lut_swizzle(pat & 0xffffu)];
        total[s] += qrow[si0];
        same_cnt += si0 == 0 ? 1u : 0u;
        if (pair) {
          const uint32_t si1 = s_sel[lut_swizzle(pat >> 16)];
          total[s] += qrow[n_combo + si1];
          same_cnt += si1 == 0 ? 1u : 0u;
        }
        // about 32 look-ups in flight at a time: more only costs registers
        if ((s + 1) % (NIB <= 4 ? 8 : 4) == 0) __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
#pragma unroll
  for (int s = 0; s < SPL; ++s) {
    const uint32_t sub = (blockIdx.x * SPL + s) * 256 + tid;
    if (sub < n_sub) {
      partial[(int64_t)blockIdx.y * n_sub + sub] = total[s];
      partial_cnt[(int64_t)blockIdx.y * n_sub + sub] = (s == 0 && count_same) ? same_cnt : 0u;   // only the sum is used
    }
  }
}

// ------------------------------------------------------------------ reduce + argmin
__global__ __launch_bounds__(256) void zero_i64_kernel(unsigned long long* p) { *p = 0ull; }

// A workgroup adds the partial sums of SUBS neighbouring subsets: thread (strand, j) adds tiles strand,
// strand + 256 / SUBS, ... of subset j in fp64, then a tree over the strands; the order depends on nothing but
// the tile count and SUBS.  SUBS = 1 suits a handful of subsets; with thousands, SUBS = 32 reads the partial
// sums (subset index fastest) in 128-byte runs.
template <int SUBS>
__global__ __launch_bounds__(256) void reduce_kernel(const float* __restrict__ partial,
                                                     const uint32_t* __restrict__ partial_cnt,
                                                     int64_t n_tiles, uint32_t n_sub,
                                                     float* __restrict__ loss,
                                                     unsigned long long* unaffected) {
  constexpr int STRANDS = 256 / SUBS;
  __shared__ double ss[256];
  __shared__ unsigned long long sc[256];
  const int j = threadIdx.x % SUBS, strand = threadIdx.x / SUBS;
  const uint32_t sub = blockIdx.x * SUBS + j;
  double s = 0.0;
  unsigned long long c = 0;
  if (sub < n_sub)
    for (int64_t i = strand; i < n_tiles; i += STRANDS) {
      s += (double)partial[i * n_sub + sub];
      c += partial_cnt[i * n_sub + sub];
    }
  ss[threadIdx.x] = s;
  sc[threadIdx.x] = c;
  __syncthreads();
  for (int off = STRANDS / 2; off >= 1; off >>= 1) {
    if (strand < off) {
      ss[threadIdx.x] += ss[threadIdx.x + off * SUBS];
      sc[threadIdx.x] += sc[threadIdx.x + off * SUBS];
    }
    __syncthreads();
  }
  if (strand == 0 && sub < n_sub) {
    loss[sub] = (float)ss[threadIdx.x];
    if (unaffected && sc[threadIdx.x]) atomicAdd(unaffected, sc[threadIdx.x]);   // integer: order does not matter
  }
}

__global__ __launch_bounds__(1024) void argmin_kernel(const float* __restrict__ loss,
                                                      uint32_t n_sub, int E, int r,
                                                      int32_t* argmin, uint32_t* argmin_mask) {
  __shared__ float sv[1024];
  __shared__ uint32_t si[1024];
  float best = INFINITY;
  uint32_t bi = 0xffffffffu;
  for (uint32_t i = threadIdx.x; i < n_sub; i += 1024) {
    const float v = loss[i];
    if (v < best || bi == 0xffffffffu) { best = v; bi = i; }   // ascending i: first minimum wins
  }
  sv[threadIdx.x] = best;
  si[threadIdx.x] = bi;
  __syncthreads();
  for (int off = 512; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off) {
      const float v = sv[threadIdx.x + off];
      const uint32_t i = si[threadIdx.x + off];
      const float mv = sv[threadIdx.x];
      const uint32_t mi = si[threadIdx.x];
      if (i != 0xffffffffu && (mi == 0xffffffffu || v < mv || (v == mv && i < mi))) {
        sv[threadIdx.x] = v;
        si[threadIdx.x] = i;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const uint32_t i = si[0] == 0xffffffffu ? 0u : si[0];
    *argmin = (int32_t)i;
    *argmin_mask = unrank_device(E, r, i);
  }
}

// Lanes per scoring workgroup: one lane per subset, whole wavefronts, at most four of them.
int score_threads(int64_t n_sub) {
  return n_sub >= 256 ? 256 : (int)((n_sub + 63) / 64) * 64;
}

int capacity_for(int n_act) {
  const int caps[] = {2, 4, 6, 8, 12, 16, 32};
  for (int c : caps)
    if (n_act <= c) return c;
  return -1;
}

}  // namespace

int plan_enumerate(int64_t T, int E, int H, int k, int r, EnumPlan* p) {
  if (k < 1 || k > E) return fail(MOEP_EINVAL, "prune_enumerate: k=%d out of range [1, E=%d]", k, E);
  if (r < 1 || r > E) return fail(MOEP_EINVAL, "prune_enumerate: r=%d out of range [1, E=%d]", r, E);
  p->T = T; p->E = E; p->H = H; p->k = k; p->r = r;
  p->kk = k < r ? k : r;
  const int n_act = p->kk + E - r;
  p->n_act = n_act < E ? n_act : E;
  p->n_sub = binomial(E, r);
  if (p->n_sub > ((int64_t)1 << 24))
    return fail(MOEP_EUNSUPPORTED, "prune_enumerate: C(%d,%d) = %lld subsets exceeds 2^24", E, r, (long long)p->n_sub);
  const int cap = capacity_for(p->n_act);
  p->rec_floats = rec_size(cap);
  // With many subsets and few possible selections per token, score through per-token selection tables.
  const int64_t n_combo = binomial(p->n_act, p->kk);
  p->n_combo = (int)(n_combo < (1 << 20) ? n_combo : (1 << 20));
  p->use_lut = p->n_sub >= 512 && p->n_act <= LUT_MAX_ACT && n_combo <= LUT_MAX_COMBO;
  p->lut_spl = 0;
  if (p->use_lut) {
    // Subsets per lane: the choice that leaves the fewest idle slots in the last workgroup of 256 lanes, among those
    // whose look-up addresses (one per subset and mask nibble, the same for every token) fit the register file.
    int64_t best = 0;
    for (int spl : {8, 17}) {
      if (spl > 8 && spl * ((E + 3) / 4) > LUT_MAX_ADDR) continue;
      const int64_t slots = ceil_div(p->n_sub, 256 * spl) * spl;
      if (!p->lut_spl || slots < best) { p->lut_spl = spl; best = slots; }
    }
    // Workgroups of equal length, about as many as a 256-CU part holds at once (three per CU by their LDS): tiles
    // of whole token groups, 32 to 1024 tokens.
    const int64_t sub_blocks = ceil_div(p->n_sub, 256 * p->lut_spl);
    const int64_t want_tiles = sub_blocks < 768 ? 768 / sub_blocks : 1;
    int64_t tile = ceil_div(ceil_div(T, want_tiles), LUT_TG) * LUT_TG;
    tile = tile < 32 ? 32 : tile > 1024 ? 1024 : tile;
    p->tok_tile = (int)tile;
  } else {
    // Aim for a few thousand scoring workgroups; tiles of 32..256 tokens.
    const int64_t sub_blocks = ceil_div(p->n_sub, score_threads(p->n_sub));
    int tile = 256;
    while (tile > 32 && sub_blocks * ceil_div(T, tile) < 4096) tile >>= 1;
    p->tok_tile = tile;
  }
  p->n_tok_tiles = ceil_div(T, p->tok_tile);
  if (p->n_tok_tiles > 65535) {                          // the grid's second dimension
    p->tok_tile = (int)(ceil_div(ceil_div(T, 65535), LUT_TG) * LUT_TG);
    p->n_tok_tiles = ceil_div(T, p->tok_tile);
  }
  size_t off = 0;
  p->off_gram = off; off += align256((size_t)T * E * E * sizeof(float));
  p->off_rec = off; off += align256((size_t)T * p->rec_floats * sizeof(float));
  p->off_masks = off;
  p->off_partial = off; off += align256((size_t)p->n_tok_tiles * p->n_sub * sizeof(float));
  p->off_partial_cnt = off; off += align256((size_t)p->n_tok_tiles * p->n_sub * sizeof(uint32_t));
  p->off_qtab = p->off_sel = p->off_selbits = p->off_nib = off;
  if (p->use_lut) {
    p->off_qtab = off; off += align256((size_t)T * p->n_combo * sizeof(float));
    p->off_sel = off; off += align256(((size_t)1 << p->n_act) * sizeof(uint16_t));
    p->off_selbits = off; off += align256((size_t)p->n_combo * sizeof(uint16_t));
    p->off_nib = off; off += align256((size_t)((T + 1) / 2) * ((E + 3) / 4) * 16 * sizeof(uint32_t));
  }
  p->total = off > 0 ? off : 256;
  return MOEP_OK;
}

template <int CAP>
static void launch_score(const EnumPlan& p, const float* rec, float* partial, uint32_t* pcnt,
                         hipStream_t s) {
  const int threads = score_threads(p.n_sub);
  dim3 grid((unsigned)ceil_div(p.n_sub, threads), (unsigned)p.n_tok_tiles);
  if (p.n_act == CAP)
    hipLaunchKernelGGL((score_kernel<CAP, true>), grid, dim3(threads), 0, s, rec, p.T, p.tok_tile, p.E, p.r,
                       p.kk, p.k, p.n_act, (uint32_t)p.n_sub, partial, pcnt);
  else
    hipLaunchKernelGGL((score_kernel<CAP, false>), grid, dim3(threads), 0, s, rec, p.T, p.tok_tile, p.E, p.r,
                       p.kk, p.k, p.n_act, (uint32_t)p.n_sub, partial, pcnt);
}

int launch_enumerate(const EnumPlan& p, const float* logits, const void* Y, moep_dtype dt,
                     float* loss, int32_t* argmin, uint32_t* argmin_mask, int64_t* unaffected,
                     char* ws, hipStream_t s, const RankedSource* ranked, bool reuse_gram) {
  float* G = (float*)(ws + p.off_gram);
  float* rec = (float*)(ws + p.off_rec);
  float* partial = (float*)(ws + p.off_partial);
  uint32_t* pcnt = (uint32_t*)(ws + p.off_partial_cnt);
  const int cap = capacity_for(p.n_act);
  if (p.T > 0) {
    // The Gram matrices do not depend on r: a caller that scores several r on the same logits and Y (and the same
    // workspace: G sits at its start whatever r is) computes them once.
    if (!reuse_gram) {
      Timed t("gram", s);
      const unsigned per_tok_blocks = (unsigned)ceil_div(p.T, 4);
      // streaming loads for a Y beyond half a GB
      const bool stream = (double)p.T * (ranked ? ranked->n_rank : p.E) * p.H * 2.0 >= 512.0 * 1024 * 1024;
#define MOEP_GRAM_LAUNCH(EPAD, RANKED, GRID, ...)                                                              \
  do {                                                                                                         \
    if (stream)                                                                                                \
      hipLaunchKernelGGL((gram_bf16_kernel<EPAD, RANKED, true>), dim3(GRID), dim3(256), 0, s, __VA_ARGS__);    \
    else                                                                                                       \
      hipLaunchKernelGGL((gram_bf16_kernel<EPAD, RANKED, false>), dim3(GRID), dim3(256), 0, s, __VA_ARGS__);   \
  } while (0)
      if (ranked) {
        const int n = ranked->n_rank;
        if (dt != MOEP_BF16)
          hipLaunchKernelGGL(gram_ranked_f32_kernel, dim3(per_tok_blocks), dim3(256), 0, s, (const float*)Y,
                             ranked->slot_of, ranked->experts, G, p.T, p.E, n, p.H);
        else if (n <= 4)
          MOEP_GRAM_LAUNCH(4, true, (unsigned)ceil_div(p.T, 16), (const uint4*)Y, ranked->slot_of, ranked->experts, G,
                           p.T, p.E, n, p.H);
        else if (n <= 8)
          MOEP_GRAM_LAUNCH(8, true, (unsigned)ceil_div(p.T, 8), (const uint4*)Y, ranked->slot_of, ranked->experts, G,
                           p.T, p.E, n, p.H);
        else
          MOEP_GRAM_LAUNCH(16, true, per_tok_blocks, (const uint4*)Y, ranked->slot_of, ranked->experts, G, p.T, p.E, n,
                           p.H);
      } else if (dt == MOEP_BF16) {
        if (p.E <= 4)
          MOEP_GRAM_LAUNCH(4, false, (unsigned)ceil_div(p.T, 16), (const uint4*)Y, nullptr, nullptr, G, p.T, p.E, 0, p.H);
        else if (p.E <= 8)
          MOEP_GRAM_LAUNCH(8, false, (unsigned)ceil_div(p.T, 8), (const uint4*)Y, nullptr, nullptr, G, p.T, p.E, 0, p.H);
        else if (p.E <= 16)
          MOEP_GRAM_LAUNCH(16, false, per_tok_blocks, (const uint4*)Y, nullptr, nullptr, G, p.T, p.E, 0, p.H);
        else
          hipLaunchKernelGGL(gram_bf16_32_kernel, dim3(per_tok_blocks), dim3(256), 0, s, (const uint4*)Y, G, p.T, p.E, p.H);
#undef MOEP_GRAM_LAUNCH
      } else {
        hipLaunchKernelGGL(gram_f32_kernel, dim3(per_tok_blocks), dim3(256), 0, s, (const float*)Y, G, p.T, p.E, p.H);
      }
      MOEP_HIP(hipGetLastError());
    }
    {
      Timed t("routing_prep", s);
      // threads (= tokens) per workgroup: as many as fit 64 KB of LDS with their records, 64 at least
      int tpb = 256;
      while (tpb > 64 && (size_t)(p.rec_floats + 1) * tpb * sizeof(float) > 64 * 1024) tpb >>= 1;
      const size_t lds = (size_t)(p.rec_floats + 1) * tpb * sizeof(float);
      const bool staged = lds <= 64 * 1024;
      if (!staged) tpb = 256;
      const dim3 grid((unsigned)ceil_div(p.T, tpb));
#define MOEP_PREP_LAUNCH(EMAX)                                                                                      \
  do {                                                                                                              \
    if (staged)                                                                                                     \
      hipLaunchKernelGGL((prep_kernel<EMAX, true>), grid, dim3(tpb), lds, s, logits, G, rec, p.T, p.E, p.k, p.n_act, \
                         cap, p.rec_floats);                                                                        \
    else                                                                                                            \
      hipLaunchKernelGGL((prep_kernel<EMAX, false>), grid, dim3(tpb), 0, s, logits, G, rec, p.T, p.E, p.k, p.n_act,  \
                         cap, p.rec_floats);                                                                        \
  } while (0)
      if (p.E <= 8) MOEP_PREP_LAUNCH(8);
      else if (p.E <= 16) MOEP_PREP_LAUNCH(16);
      else MOEP_PREP_LAUNCH(32);
#undef MOEP_PREP_LAUNCH
      MOEP_HIP(hipGetLastError());
    }
    if (p.use_lut) {
      Timed t("subset_score_tables", s);
      float* qtab = (float*)(ws + p.off_qtab);
      uint16_t* sel = (uint16_t*)(ws + p.off_sel);
      uint16_t* selbits = (uint16_t*)(ws + p.off_selbits);
      hipLaunchKernelGGL(selidx_kernel, dim3((unsigned)ceil_div((int64_t)1 << p.n_act, 256)), dim3(256), 0, s, p.n_act,
                         p.kk, sel, selbits);
      uint16_t* nibtab = (uint16_t*)(ws + p.off_nib);
      const int nib = (p.E + 3) / 4;
      const dim3 qgrid((unsigned)p.T), qblock(p.n_combo <= 64 ? 64 : 256);
#define MOEP_QTABLE_CASE(C)                                                                                       \
  case C:                                                                                                         \
    if (p.n_act == C)                                                                                             \
      hipLaunchKernelGGL((qtable_kernel<C, true>), qgrid, qblock, 0, s, rec, p.kk, p.k, p.n_act, p.n_combo,       \
                         selbits, qtab, nib, nibtab);                                                             \
    else                                                                                                          \
      hipLaunchKernelGGL((qtable_kernel<C, false>), qgrid, qblock, 0, s, rec, p.kk, p.k, p.n_act, p.n_combo,      \
                         selbits, qtab, nib, nibtab);                                                             \
    break;
      switch (cap) {
        MOEP_QTABLE_CASE(2) MOEP_QTABLE_CASE(4) MOEP_QTABLE_CASE(6) MOEP_QTABLE_CASE(8) MOEP_QTABLE_CASE(12)
        default: return fail(MOEP_EUNSUPPORTED, "prune_enumerate: no selection table for %d active ranks", p.n_act);
      }
#undef MOEP_QTABLE_CASE
      const dim3 grid((unsigned)ceil_div(p.n_sub, 256 * p.lut_spl), (unsigned)p.n_tok_tiles);
      const bool count_same = p.kk == p.k;
#define MOEP_LUT_LAUNCH(N, S)                                                                                     \
  hipLaunchKernelGGL((score_lut_kernel<N, S>), grid, dim3(256), 0, s, qtab, (const uint32_t*)nibtab, sel, p.T, p.tok_tile, p.E,    \
                     p.r, p.n_act, p.n_combo, count_same, (uint32_t)p.n_sub, partial, pcnt)
      // 512 subsets or more with at most 12 active ranks: 12 experts at least, three nibbles
      switch (nib * 100 + p.lut_spl) {
        case 308: MOEP_LUT_LAUNCH(3, 8); break;
        case 408: MOEP_LUT_LAUNCH(4, 8); break;
        case 417: MOEP_LUT_LAUNCH(4, 17); break;         // (up to 12 experts never have the subsets for it)
        case 508: MOEP_LUT_LAUNCH(5, 8); break;
        case 608: MOEP_LUT_LAUNCH(6, 8); break;
        case 708: MOEP_LUT_LAUNCH(7, 8); break;
        case 808: MOEP_LUT_LAUNCH(8, 8); break;
        default:
          return fail(MOEP_EUNSUPPORTED, "prune_enumerate: no table scorer for %d experts, %d subsets per lane", p.E,
                      p.lut_spl);
      }
#undef MOEP_LUT_LAUNCH
      MOEP_HIP(hipGetLastError());
    } else {
      Timed t("subset_score", s);
      switch (cap) {
        case 2: launch_score<2>(p, rec, partial, pcnt, s); break;
        case 4: launch_score<4>(p, rec, partial, pcnt, s); break;
        case 6: launch_score<6>(p, rec, partial, pcnt, s); break;
        case 8: launch_score<8>(p, rec, partial, pcnt, s); break;
        case 12: launch_score<12>(p, rec, partial, pcnt, s); break;
        case 16: launch_score<16>(p, rec, partial, pcnt, s); break;
        case 32: launch_score<32>(p, rec, partial, pcnt, s); break;
        default: return fail(MOEP_EUNSUPPORTED, "prune_enumerate: no scorer for %d active ranks", p.n_act);
      }
      MOEP_HIP(hipGetLastError());
    }
  }
  return launch_reduce_argmin(partial, pcnt, p.T > 0 ? p.n_tok_tiles : 0, p.n_sub, p.E, p.r, loss, argmin, argmin_mask,
                              unaffected, s);
}

int launch_reduce_argmin(const float* partial, const uint32_t* pcnt, int64_t n_tiles, int64_t n_sub, int E, int r,
                         float* loss, int32_t* argmin, uint32_t* argmin_mask, int64_t* unaffected, hipStream_t s) {
  Timed t("loss_reduce_argmin", s);
  if (unaffected) hipLaunchKernelGGL(zero_i64_kernel, dim3(1), dim3(1), 0, s, (unsigned long long*)unaffected);
  if (n_sub >= 1024)
    hipLaunchKernelGGL(reduce_kernel<32>, dim3((unsigned)ceil_div(n_sub, 32)), dim3(256), 0, s, partial, pcnt,
                       n_tiles, (uint32_t)n_sub, loss, (unsigned long long*)unaffected);
  else
    hipLaunchKernelGGL(reduce_kernel<1>, dim3((unsigned)n_sub), dim3(256), 0, s, partial, pcnt, n_tiles,
                       (uint32_t)n_sub, loss, (unsigned long long*)unaffected);
  hipLaunchKernelGGL(argmin_kernel, dim3(1), dim3(1024), 0, s, loss, (uint32_t)n_sub, E, r, argmin, argmin_mask);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

int launch_subset_masks(int E, int r, int64_t n_sub, uint32_t* masks, hipStream_t s) {
  hipLaunchKernelGGL(masks_kernel, dim3((unsigned)ceil_div(n_sub, 256)), dim3(256), 0, s, E, r, (uint32_t)n_sub, masks);
  MOEP_HIP(hipGetLastError());
  return MOEP_OK;
}

}  // namespace moep
