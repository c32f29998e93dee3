// Host side of libmoeprune: the C ABI declared in include/moeprune.h.
// Argument checks, subset rank/unrank, workspace carving, per-kernel timing and the
// sequencing of kernel launches.  No arithmetic of the method runs here.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "common.h"

namespace moep {

// ---------------------------------------------------------------- errors
static thread_local char g_err[512] = "";

int fail(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return status;
}

// ---------------------------------------------------------------- subsets
int64_t binomial(int n, int r) {
  if (r < 0 || r > n) return 0;
  if (r > n - r) r = n - r;
  int64_t c = 1;
  for (int i = 1; i <= r; ++i) c = c * (n - r + i) / i;   // exact: c is C(n-r+i, i) after step i
  return c;
}

// Lexicographic unranking of sorted r-tuples over {0..E-1}: walking the experts in
// ascending order, C(E-1-e, rem-1) subsets put e as their next smallest element.
uint32_t unrank_mask(int E, int r, int64_t idx) {
  uint32_t mask = 0;
  int rem = r;
  for (int e = 0; e < E && rem > 0; ++e) {
    int64_t with_e = binomial(E - 1 - e, rem - 1);
    if (idx < with_e) { mask |= 1u << e; --rem; }
    else idx -= with_e;
  }
  return mask;
}

// ---------------------------------------------------------------- timing
namespace {
struct TimingState {
  std::mutex mu;
  bool on = false;
  struct Rec { const char* name; hipEvent_t start, stop; bool used; };
  std::vector<Rec> pool;      // events created once, on enable
  int next = 0;
};
TimingState g_timing;
constexpr int kMaxTimed = 8192;
}  // namespace

Timed::Timed(const char* kernel_name, hipStream_t s) : slot(-1), stream(s) {
  TimingState& t = g_timing;
  if (!t.on) return;
  std::lock_guard<std::mutex> lk(t.mu);
  if (!t.on || t.next >= (int)t.pool.size()) return;
  slot = t.next++;
  t.pool[slot].name = kernel_name;
  t.pool[slot].used = true;
  (void)hipEventRecord(t.pool[slot].start, stream);
}

Timed::~Timed() {
  if (slot < 0) return;
  (void)hipEventRecord(g_timing.pool[slot].stop, stream);
}

static bool valid_shape(int64_t T, int E, int H, int F, moep_dtype dt, const char* who) {
  if (dt != MOEP_F32 && dt != MOEP_BF16) { fail(MOEP_EINVAL, "%s: unknown dtype %d", who, (int)dt); return false; }
  if (T < 0 || T > (int64_t)1 << 30) { fail(MOEP_EINVAL, "%s: T=%lld out of range [0, 2^30]", who, (long long)T); return false; }
  if (E < 1 || E > 32) { fail(MOEP_EINVAL, "%s: E=%d out of range [1, 32]", who, E); return false; }
  if (H < 1 || (F < 1)) { fail(MOEP_EINVAL, "%s: H=%d, F=%d must be positive", who, H, F); return false; }
  return true;
}

static int check_alignment(int H, int F, moep_dtype dt, const char* who) {
  int q = dt == MOEP_BF16 ? 64 : 4;
  if (H % q || F % q)
    return fail(MOEP_EUNSUPPORTED, "%s: H=%d and F=%d must be multiples of %d for this dtype", who, H, F, q);
  if ((int64_t)H > 65536 || (int64_t)F > 262144)
    return fail(MOEP_EUNSUPPORTED, "%s: H=%d or F=%d beyond the supported maximum", who, H, F);
  return MOEP_OK;
}

static int check_ws(const void* ws, size_t ws_bytes, size_t need, const char* who) {
  if (need == 0) return MOEP_OK;
  if (!ws) return fail(MOEP_EWORKSPACE, "%s: workspace is NULL, %zu bytes needed", who, need);
  if ((uintptr_t)ws & 255) return fail(MOEP_EWORKSPACE, "%s: workspace must be 256-byte aligned", who);
  if (ws_bytes < need) return fail(MOEP_EWORKSPACE, "%s: workspace has %zu bytes, %zu needed", who, ws_bytes, need);
  return MOEP_OK;
}


}  // namespace moep

using namespace moep;

extern "C" {

const char* moep_last_error(void) { return g_err; }

int64_t moep_num_subsets(int E, int r) {
  if (E < 1 || E > 32 || r < 1 || r > E) return -1;
  return binomial(E, r);
}

int moep_subset_unrank(int E, int r, int64_t idx, uint32_t* mask_out) {
  int64_t n = moep_num_subsets(E, r);
  if (n < 0) return fail(MOEP_EINVAL, "moep_subset_unrank: need 1 <= r <= E <= 32 (E=%d, r=%d)", E, r);
  if (!mask_out) return fail(MOEP_EINVAL, "moep_subset_unrank: mask_out is NULL");
  if (idx < 0 || idx >= n) return fail(MOEP_EINVAL, "moep_subset_unrank: index %lld not in [0, %lld)", (long long)idx, (long long)n);
  *mask_out = unrank_mask(E, r, idx);
  return MOEP_OK;
}

int64_t moep_subset_rank(int E, int r, uint32_t mask) {
  if (moep_num_subsets(E, r) < 0) return -1;
  if (E < 32 && (mask >> E)) return -1;
  if (__builtin_popcount(mask) != r) return -1;
  int64_t idx = 0;
  int rem = r;
  for (int e = 0; e < E && rem > 0; ++e) {
    if (mask & (1u << e)) --rem;
    else idx += binomial(E - 1 - e, rem - 1);   // all subsets whose next element is e come first
  }
  return idx;
}

// ------------------------------------------------------------------ timing
int moep_timing_enable(int on) {
  TimingState& t = g_timing;
  std::lock_guard<std::mutex> lk(t.mu);
  if (on && t.pool.empty()) {
    t.pool.resize(kMaxTimed);
    for (auto& r : t.pool) {
      r.used = false;
      r.name = nullptr;
      if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) {
        t.pool.clear();
        return fail(MOEP_EHIP, "moep_timing_enable: hipEventCreate failed");
      }
    }
  }
  t.on = on != 0;
  return MOEP_OK;
}

int moep_timing_collect(const char** names, double* total_ms, int64_t* launches, int cap) {
  TimingState& t = g_timing;
  std::lock_guard<std::mutex> lk(t.mu);
  if (!names || !total_ms || !launches || cap <= 0) {
    fail(MOEP_EINVAL, "moep_timing_collect: NULL array or cap <= 0");
    return -1;
  }
  int n = 0;
  for (int i = 0; i < t.next; ++i) {
    auto& r = t.pool[i];
    if (!r.used) continue;
    r.used = false;
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
      fail(MOEP_EHIP, "moep_timing_collect: event query failed for %s", r.name);
      t.next = 0;
      return -1;
    }
    int j = 0;
    while (j < n && strcmp(names[j], r.name) != 0) ++j;
    if (j == n) {
      if (n == cap) continue;
      names[n] = r.name; total_ms[n] = 0.0; launches[n] = 0; ++n;
    }
    total_ms[j] += ms;
    launches[j] += 1;
  }
  t.next = 0;
  return n;
}

int moep_timing_records(const char** names, float* ms, int cap) {
  TimingState& t = g_timing;
  std::lock_guard<std::mutex> lk(t.mu);
  if (!names || !ms || cap <= 0) {
    fail(MOEP_EINVAL, "moep_timing_records: NULL array or cap <= 0");
    return -1;
  }
  int n = 0;
  for (int i = 0; i < t.next; ++i) {
    auto& r = t.pool[i];
    if (!r.used) continue;
    r.used = false;
    float v = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&v, r.start, r.stop) != hipSuccess) {
      fail(MOEP_EHIP, "moep_timing_records: event query failed for %s", r.name);
      t.next = 0;
      return -1;
    }
    if (n < cap) { names[n] = r.name; ms[n] = v; ++n; }
  }
  t.next = 0;
  return n;
}

// ------------------------------------------------------------------ moe_expert_outputs
// bf16: how many experts go into one launch of each projection.  One launch per projection over ALL experts
// saves the fill and drain of the persistent kernel per expert (what matters when a launch takes a
// millisecond or two), at the price of holding every expert's h at once; beyond kBatchedHBytes of h the
// experts are taken in batches that fit.
static constexpr size_t kBatchedHBytes = (size_t)12 << 30;
static int experts_per_launch(int64_t T, int E, int F) {
  const size_t per = packed_a_bytes(T, F);
  if (per == 0) return E;
  const size_t fit = kBatchedHBytes / per;
  return fit < 1 ? 1 : (fit > (size_t)E ? E : (int)fit);
}

static size_t expert_outputs_workspace_bf16(int64_t T, int E, int H, int F, bool weights_prepacked) {
  size_t need = align256((size_t)experts_per_launch(T, E, F) * packed_a_bytes(T, F)) + align256(packed_a_bytes(T, H));
  if (!weights_prepacked)
    need += align256((size_t)E * packed_b_bytes(F, H, true)) + align256((size_t)E * packed_b_bytes(H, F, false));
  return need;
}

size_t moe_expert_outputs_workspace(int64_t T, int E, int H, int F, moep_dtype dt) {
  if (!valid_shape(T, E, H, F, dt, "moe_expert_outputs_workspace")) return 0;
  if (dt == MOEP_BF16)   // packed h of one batch of experts, packed x, every expert's packed W1/W3 pair and packed W2
    return expert_outputs_workspace_bf16(T, E, H, F, false);
  return align256((size_t)T * (size_t)F * dtype_size(dt));
}

size_t moe_expert_outputs_packed_workspace(int64_t T, int E, int H, int F, moep_dtype dt) {
  if (!valid_shape(T, E, H, F, dt, "moe_expert_outputs_packed_workspace")) return 0;
  if (dt != MOEP_BF16 || check_alignment(H, F, dt, "moe_expert_outputs_packed_workspace")) return 0;
  return expert_outputs_workspace_bf16(T, E, H, F, true);
}

// `packed` != NULL: the expert weights as re-laid out by moe_pack_weights (W1, W3, W2 are not read).
static int expert_outputs(const void* x, const void* Wgate, const void* W1, const void* W3, const void* W2,
                          const void* packed, int64_t T, int E, int H, int F, moep_dtype dt, float* logits,
                          void* Y, void* ws, size_t ws_bytes, void* hip_stream, const char* who) {
  if (!valid_shape(T, E, H, F, dt, who)) return MOEP_EINVAL;
  if (int st = check_alignment(H, F, dt, who)) return st;
  if (packed && dt != MOEP_BF16) return fail(MOEP_EUNSUPPORTED, "%s: packed weights exist for bf16 only", who);
  if (!Wgate || (!packed && (!W1 || !W3 || !W2))) return fail(MOEP_EINVAL, "%s: NULL weight pointer", who);
  if (T == 0) return MOEP_OK;
  if (!x || !logits || !Y) return fail(MOEP_EINVAL, "%s: NULL x, logits or Y", who);
  const size_t need = dt == MOEP_BF16 ? expert_outputs_workspace_bf16(T, E, H, F, packed != nullptr)
                                      : moe_expert_outputs_workspace(T, E, H, F, dt);
  if (int st = check_ws(ws, ws_bytes, need, who)) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  const size_t es = dtype_size(dt);

  if (dt == MOEP_BF16) {
    // Operands are packed once per call into the blocked layout of the packed GEMM (x; every expert's
    // weights, unless the caller has done that already); h stays in that layout between the two projections
    // and never exists row-major.  Each projection is ONE launch over a batch of experts.
    const int eb = experts_per_launch(T, E, F);
    const size_t h_bytes = packed_a_bytes(T, F);
    char* hp = (char*)ws;
    char* xp = hp + align256((size_t)eb * h_bytes);
    const char* wgu = xp + align256(packed_a_bytes(T, H));
    const char* wdn = wgu + align256((size_t)E * packed_b_bytes(F, H, true));
    // one pass over x for the router logits and its packed copy where a fused kernel exists
    int st_x = launch_router_and_pack_x(x, Wgate, T, E, H, logits, xp, s);
    if (st_x == MOEP_EUNSUPPORTED) {
      if (int st = launch_router(x, Wgate, T, E, H, dt, logits, s)) return st;
      st_x = launch_pack_a_bf16(x, H, T, H, xp, s, "pack_x");
    }
    if (st_x) return st_x;
    if (packed) {                     // all W1/W3 pairs, then all W2
      wgu = (const char*)packed;
      wdn = wgu + (size_t)E * packed_b_bytes(F, H, true);
    } else {
      if (int st = launch_pack_b_bf16(W1, W3, F, H, E, (void*)wgu, s, "pack_w")) return st;
      if (int st = launch_pack_b_bf16(W2, nullptr, H, F, E, (void*)wdn, s, "pack_w")) return st;
    }
    for (int e0 = 0; e0 < E; e0 += eb) {
      const int ne = E - e0 < eb ? E - e0 : eb;
      PackedGemmArgs up;                          // h[e] = silu(x W1[e]^T) * (x W3[e]^T)
      up.A = xp; up.B = wgu + (size_t)e0 * packed_b_bytes(F, H, true); up.C = hp;
      up.M = T; up.N = F; up.K = H; up.epilogue = EPI_SWIGLU;
      up.experts = ne; up.a_expert_bytes = 0; up.c_expert_bytes = (int64_t)h_bytes;
      if (int st = launch_gemm_bf16_packed(up, s, "gemm_gate_up_swiglu")) return st;
      PackedGemmArgs down;                        // Y[e] = h[e] W2[e]^T
      down.A = hp; down.B = wdn + (size_t)e0 * packed_b_bytes(H, F, false);
      down.C = (char*)Y + (size_t)e0 * T * H * es; down.ldc = H;
      down.M = T; down.N = H; down.K = F; down.epilogue = EPI_STORE;
      down.experts = ne; down.a_expert_bytes = (int64_t)h_bytes; down.c_expert_bytes = (int64_t)((size_t)T * H * es);
      if (int st = launch_gemm_bf16_packed(down, s, "gemm_down")) return st;
    }
    return MOEP_OK;
  }
  if (int st = launch_router(x, Wgate, T, E, H, dt, logits, s)) return st;
  for (int e = 0; e < E; ++e) {
    GemmArgs up;                                  // h = silu(x W1[e]^T) * (x W3[e]^T)
    up.A = x; up.lda = H;
    up.B0 = (const char*)W1 + (size_t)e * F * H * es;
    up.B1 = (const char*)W3 + (size_t)e * F * H * es;
    up.C = ws; up.ldc = F;
    up.M = T; up.N = F; up.K = H;
    up.epilogue = EPI_SWIGLU;
    if (int st = launch_gemm_f32(up, s, "gemm_gate_up_swiglu")) return st;
    GemmArgs down;                                // Y[e] = h W2[e]^T
    down.A = ws; down.lda = F;
    down.B0 = (const char*)W2 + (size_t)e * H * F * es;
    down.C = (char*)Y + (size_t)e * T * H * es; down.ldc = H;
    down.M = T; down.N = H; down.K = F;
    down.epilogue = EPI_STORE;
    if (int st = launch_gemm_f32(down, s, "gemm_down")) return st;
  }
  return MOEP_OK;
}

int moe_expert_outputs(const void* x, const void* Wgate, const void* W1, const void* W3,
                       const void* W2, int64_t T, int E, int H, int F, moep_dtype dt,
                       float* logits, void* Y, void* ws, size_t ws_bytes, void* hip_stream) {
  return expert_outputs(x, Wgate, W1, W3, W2, nullptr, T, E, H, F, dt, logits, Y, ws, ws_bytes, hip_stream,
                        "moe_expert_outputs");
}

int moe_expert_outputs_packed(const void* x, const void* Wgate, const void* packed_weights, int64_t T, int E,
                              int H, int F, moep_dtype dt, float* logits, void* Y, void* ws, size_t ws_bytes,
                              void* hip_stream) {
  if (!packed_weights) return fail(MOEP_EINVAL, "moe_expert_outputs_packed: packed_weights is NULL");
  return expert_outputs(x, Wgate, nullptr, nullptr, nullptr, packed_weights, T, E, H, F, dt, logits, Y, ws,
                        ws_bytes, hip_stream, "moe_expert_outputs_packed");
}

// ------------------------------------------------------------------ prune_enumerate
size_t prune_enumerate_workspace(int64_t T, int E, int H, int k, int r, moep_dtype dt) {
  if (!valid_shape(T, E, H, 1, dt, "prune_enumerate_workspace")) return 0;
  EnumPlan p;
  if (plan_enumerate(T, E, H, k, r, &p)) return 0;
  return p.total;
}

int prune_enumerate(const float* logits, const void* Y, int64_t T, int E, int H, moep_dtype dt,
                    int k, int r, float* loss, int32_t* argmin, uint32_t* argmin_mask,
                    int64_t* unaffected_pairs, void* ws, size_t ws_bytes, void* hip_stream) {
  const char* who = "prune_enumerate";
  if (!valid_shape(T, E, H, 1, dt, who)) return MOEP_EINVAL;
  EnumPlan p;
  if (int st = plan_enumerate(T, E, H, k, r, &p)) return st;
  if (H % (dt == MOEP_BF16 ? 64 : 1))
    return fail(MOEP_EUNSUPPORTED, "%s: H=%d must be a multiple of 64 for bf16", who, H);
  if (!loss || !argmin || !argmin_mask) return fail(MOEP_EINVAL, "%s: NULL loss, argmin or argmin_mask", who);
  if (T > 0 && (!logits || !Y)) return fail(MOEP_EINVAL, "%s: NULL logits or Y", who);
  if (int st = check_ws(ws, ws_bytes, p.total, who)) return st;
  return launch_enumerate(p, logits, Y, dt, loss, argmin, argmin_mask, unaffected_pairs,
                          (char*)ws, (hipStream_t)hip_stream);
}

// Eq. 3 as written (no Gram matrices): the alternative the Gram path is measured against.
size_t prune_enumerate_direct_workspace(int64_t T, int E, int H, int k, int r, moep_dtype dt) {
  if (!valid_shape(T, E, H, 1, dt, "prune_enumerate_direct_workspace")) return 0;
  DirectPlan p;
  if (plan_enumerate_direct(T, E, H, k, r, dt, &p)) return 0;
  return p.total;
}

int prune_enumerate_direct(const float* logits, const void* Y, int64_t T, int E, int H, moep_dtype dt, int k, int r,
                           float* loss, int32_t* argmin, uint32_t* argmin_mask, int64_t* unaffected_pairs, void* ws,
                           size_t ws_bytes, void* hip_stream) {
  const char* who = "prune_enumerate_direct";
  if (!valid_shape(T, E, H, 1, dt, who)) return MOEP_EINVAL;
  DirectPlan p;
  if (int st = plan_enumerate_direct(T, E, H, k, r, dt, &p)) return st;
  if (!loss || !argmin || !argmin_mask) return fail(MOEP_EINVAL, "%s: NULL loss, argmin or argmin_mask", who);
  if (T > 0 && (!logits || !Y)) return fail(MOEP_EINVAL, "%s: NULL logits or Y", who);
  if (int st = check_ws(ws, ws_bytes, p.total, who)) return st;
  return launch_enumerate_direct(p, logits, Y, dt, loss, argmin, argmin_mask, unaffected_pairs, (char*)ws,
                                 (hipStream_t)hip_stream);
}

// Several r on the same logits and Y: the Gram pass, which does not depend on r, runs once.
size_t prune_enumerate_multi_workspace(int64_t T, int E, int H, int k, int n_r, const int* rs, moep_dtype dt) {
  if (!valid_shape(T, E, H, 1, dt, "prune_enumerate_multi_workspace") || n_r < 1 || !rs) return 0;
  size_t need = 0;
  for (int i = 0; i < n_r; ++i) {
    EnumPlan p;
    if (plan_enumerate(T, E, H, k, rs[i], &p)) return 0;
    need = p.total > need ? p.total : need;
  }
  return need;
}

int prune_enumerate_multi(const float* logits, const void* Y, int64_t T, int E, int H, moep_dtype dt, int k,
                          int n_r, const int* rs, float* loss, int32_t* argmin, uint32_t* argmin_mask,
                          int64_t* unaffected_pairs, void* ws, size_t ws_bytes, void* hip_stream) {
  const char* who = "prune_enumerate_multi";
  if (!valid_shape(T, E, H, 1, dt, who)) return MOEP_EINVAL;
  if (n_r < 1 || !rs) return fail(MOEP_EINVAL, "%s: need at least one r", who);
  if (H % (dt == MOEP_BF16 ? 64 : 1))
    return fail(MOEP_EUNSUPPORTED, "%s: H=%d must be a multiple of 64 for bf16", who, H);
  if (!loss || !argmin || !argmin_mask) return fail(MOEP_EINVAL, "%s: NULL loss, argmin or argmin_mask", who);
  if (T > 0 && (!logits || !Y)) return fail(MOEP_EINVAL, "%s: NULL logits or Y", who);
  size_t need = 0;
  for (int i = 0; i < n_r; ++i) {            // every r is checked before anything is launched
    EnumPlan p;
    if (int st = plan_enumerate(T, E, H, k, rs[i], &p)) return st;
    need = p.total > need ? p.total : need;
  }
  if (int st = check_ws(ws, ws_bytes, need, who)) return st;
  int64_t off = 0;
  for (int i = 0; i < n_r; ++i) {
    EnumPlan p;
    plan_enumerate(T, E, H, k, rs[i], &p);
    if (int st = launch_enumerate(p, logits, Y, dt, loss + off, argmin + i, argmin_mask + i,
                                  unaffected_pairs ? unaffected_pairs + i : nullptr, (char*)ws,
                                  (hipStream_t)hip_stream, nullptr, i > 0)) return st;
    off += p.n_sub;
  }
  return MOEP_OK;
}

// ------------------------------------------------------------------ moe_forward_skip
// The two grouped GEMMs of the routed path: every slot (one routed (token, expert) pair, rows grouped
// by expert) goes through its expert, and the down projection scales it by the slot's routing weight.
// With `plain_out` the down projection instead stores the unscaled expert output of every slot there,
// in the storage dtype.
// `direct_out` (bf16 path, row-scaled mode): the layer output; slots that are a token's only one are written there.
static int run_routed_ffn(const SkipPlan& p, const void* x, const void* W1, const void* W3,
                          const void* W2, moep_dtype dt, char* w, hipStream_t s, void* plain_out = nullptr,
                          const void* packed = nullptr, void* direct_out = nullptr) {
  const int H = p.H, F = p.F;
  if (dt == MOEP_BF16) {
    // Packed-operand path: the routed rows of x are gathered into one 256-row block per tile, every
    // expert's weights are re-laid out, and h stays in the packed layout between the two projections.
    const int32_t* slot_token = (const int32_t*)(w + p.off_slot_token);
    const int32_t* tile_expert = (const int32_t*)(w + p.off_tile_expert);
    const int32_t* tile_row0 = (const int32_t*)(w + p.off_tile_row0);
    const int32_t* seg_end = (const int32_t*)(w + p.off_seg_end);
    const int32_t* tiles_in_use = tile_expert + p.max_tiles;
    if (int st = launch_pack_a_gathered_bf16(x, H, slot_token, tile_expert, tile_row0, seg_end, tiles_in_use,
                                             p.max_tiles, H, w + p.off_xp, s, "pack_x_routed")) return st;
    const char* w13 = w + p.off_w13;
    const char* w2 = w + p.off_w2;
    if (packed) {                     // packed once by moe_pack_weights: all W1/W3 pairs, then all W2
      w13 = (const char*)packed;
      w2 = w13 + (size_t)p.E * packed_b_bytes(F, H, true);
    } else {
      if (int st = launch_pack_b_bf16(W1, W3, F, H, p.E, w + p.off_w13, s, "pack_w")) return st;
      if (int st = launch_pack_b_bf16(W2, nullptr, H, F, p.E, w + p.off_w2, s, "pack_w")) return st;
    }
    PackedGemmArgs up;
    up.A = w + p.off_xp; up.B = w13; up.C = w + p.off_h;
    up.M = p.max_slots; up.N = F; up.K = H; up.epilogue = EPI_SWIGLU;
    up.tile_expert = tile_expert; up.tile_row0 = tile_row0; up.seg_end = seg_end; up.tiles_in_use = tiles_in_use;
    up.max_m_tiles = p.max_tiles;
    up.tile_order = (const uint32_t*)(w + p.off_order_up);
    if (int st = launch_gemm_bf16_packed(up, s, "gemm_gate_up_swiglu_routed")) return st;
    PackedGemmArgs down = up;
    down.tile_order = (const uint32_t*)(w + p.off_order_down);
    down.A = w + p.off_h; down.B = w2;
    down.C = plain_out ? plain_out : w + p.off_slot_out; down.ldc = H;
    down.N = H; down.K = F;
    down.epilogue = plain_out ? EPI_STORE : EPI_ROWSCALE_F32;
    down.row_scale = plain_out ? nullptr : (const float*)(w + p.off_slot_scale);
    if (!plain_out && direct_out) {
      down.row_dest = (const int32_t*)(w + p.off_slot_dest);
      down.direct_out = direct_out;
    }
    return launch_gemm_bf16_packed(down, s, "gemm_down_routed");
  }
  GemmArgs up;                      // h[slot] = silu(x[token(slot)] W1[e]^T) * (x[..] W3[e]^T)
  up.A = x; up.lda = H; up.a_rows = (const int32_t*)(w + p.off_slot_token);
  up.B0 = W1; up.B1 = W3; up.b_expert_stride = (int64_t)F * H;
  up.C = w + p.off_h; up.ldc = F;
  up.M = p.max_slots; up.N = F; up.K = H;
  up.epilogue = EPI_SWIGLU;
  up.tile_expert = (const int32_t*)(w + p.off_tile_expert);
  up.tile_row0 = (const int32_t*)(w + p.off_tile_row0);
  up.seg_end = (const int32_t*)(w + p.off_seg_end);
  up.max_m_tiles = p.max_tiles;
  up.tiles_in_use = up.tile_expert + p.max_tiles;
  if (int st = launch_gemm_f32(up, s, "gemm_gate_up_swiglu_routed")) return st;

  GemmArgs down;                    // slot_out[slot] = weight(slot) * h[slot] W2[e]^T, fp32
  down.A = w + p.off_h; down.lda = F;
  down.B0 = W2; down.b_expert_stride = (int64_t)H * F;
  down.C = plain_out ? plain_out : w + p.off_slot_out; down.ldc = H;
  down.M = p.max_slots; down.N = H; down.K = F;
  down.epilogue = plain_out ? EPI_STORE : EPI_ROWSCALE_F32;
  down.row_scale = plain_out ? nullptr : (const float*)(w + p.off_slot_scale);
  down.tile_expert = up.tile_expert; down.tile_row0 = up.tile_row0; down.seg_end = up.seg_end;
  down.max_m_tiles = p.max_tiles;
  down.tiles_in_use = up.tiles_in_use;
  return launch_gemm_f32(down, s, "gemm_down_routed");
}

size_t moe_forward_skip_workspace(int64_t T, int E, int H, int F, moep_dtype dt) {
  if (!valid_shape(T, E, H, F, dt, "moe_forward_skip_workspace")) return 0;
  SkipPlan p;
  if (plan_skip(T, E, H, F, dt, 2, &p)) return 0;
  return p.total;
}

int moe_forward_skip(const void* x, const void* Wgate, const void* W1, const void* W3,
                     const void* W2, int64_t T, int E, int H, int F, moep_dtype dt, int k,
                     float beta, void* out, uint8_t* skip_mask, float* logits_out,
                     int32_t* top2_out, void* ws, size_t ws_bytes, void* hip_stream) {
  const uint32_t all = (E >= 1 && E < 32) ? (1u << E) - 1u : 0xffffffffu;
  return moe_forward_pruned_skip(x, Wgate, W1, W3, W2, T, E, H, F, dt, k, all, beta, out, skip_mask,
                                 logits_out, top2_out, ws, ws_bytes, hip_stream);
}

// `packed` != NULL: the expert weights as re-laid out by moe_pack_weights (W1, W3, W2 are not read).
static int forward_pruned_skip(const void* x, const void* Wgate, const void* W1, const void* W3,
                               const void* W2, const void* packed, int64_t T, int E, int H, int F,
                               moep_dtype dt, int k, uint32_t kept_mask, float beta, void* out,
                               uint8_t* skip_mask, float* logits_out, int32_t* top2_out, void* ws,
                               size_t ws_bytes, void* hip_stream) {
  const char* who = "moe_forward_skip";
  if (!valid_shape(T, E, H, F, dt, who)) return MOEP_EINVAL;
  if (k != 2) return fail(MOEP_EUNSUPPORTED, "%s: only k = 2 is implemented (k=%d)", who, k);
  if (E < 2) return fail(MOEP_EINVAL, "%s: top-2 routing needs E >= 2 (E=%d)", who, E);
  if (E < 32 && (kept_mask >> E)) return fail(MOEP_EINVAL, "%s: kept_mask 0x%x has bits beyond expert %d", who, kept_mask, E - 1);
  if (__builtin_popcount(kept_mask) < 2) return fail(MOEP_EINVAL, "%s: kept_mask 0x%x keeps fewer than two experts", who, kept_mask);
  if (!(beta >= 0.0f) || std::isinf(beta)) return fail(MOEP_EINVAL, "%s: beta must be finite and >= 0", who);
  if (int st = check_alignment(H, F, dt, who)) return st;
  if (!Wgate || (!packed && (!W1 || !W3 || !W2))) return fail(MOEP_EINVAL, "%s: NULL weight pointer", who);
  if (packed && dt != MOEP_BF16) return fail(MOEP_EUNSUPPORTED, "%s: packed weights exist for bf16 only", who);
  if (T == 0) return MOEP_OK;
  if (!x || !out || !skip_mask) return fail(MOEP_EINVAL, "%s: NULL x, out or skip_mask", who);
  SkipPlan p;
  if (int st = plan_skip(T, E, H, F, dt, 2, &p)) return st;
  if (int st = check_ws(ws, ws_bytes, p.total, who)) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  char* w = (char*)ws;

  float* logits = logits_out ? logits_out : (float*)(w + p.off_logits);
  if (int st = launch_router(x, Wgate, T, E, H, dt, logits, s)) return st;
  if (int st = launch_skip_routing(p, logits, kept_mask, beta, skip_mask, top2_out, w, s)) return st;

  // bf16: the down projection writes the output of every token routed to a single expert itself
  void* direct = dt == MOEP_BF16 ? out : nullptr;
  if (int st = run_routed_ffn(p, x, W1, W3, W2, dt, w, s, nullptr, packed, direct)) return st;
  return launch_skip_combine(p, dt, skip_mask, out, w, s, direct != nullptr);
}

int moe_forward_pruned_skip(const void* x, const void* Wgate, const void* W1, const void* W3,
                            const void* W2, int64_t T, int E, int H, int F, moep_dtype dt, int k,
                            uint32_t kept_mask, float beta, void* out, uint8_t* skip_mask,
                            float* logits_out, int32_t* top2_out, void* ws, size_t ws_bytes,
                            void* hip_stream) {
  return forward_pruned_skip(x, Wgate, W1, W3, W2, nullptr, T, E, H, F, dt, k, kept_mask, beta, out, skip_mask,
                             logits_out, top2_out, ws, ws_bytes, hip_stream);
}

// ------------------------------------------------------------------ packed weights for serving loops
size_t moe_packed_weights_bytes(int E, int H, int F, moep_dtype dt) {
  if (!valid_shape(1, E, H, F, dt, "moe_packed_weights_bytes")) return 0;
  if (dt != MOEP_BF16 || check_alignment(H, F, dt, "moe_packed_weights_bytes")) return 0;
  return (size_t)E * (packed_b_bytes(F, H, true) + packed_b_bytes(H, F, false));
}

int moe_pack_weights(const void* W1, const void* W3, const void* W2, int E, int H, int F, moep_dtype dt,
                     void* packed, void* hip_stream) {
  const char* who = "moe_pack_weights";
  if (!valid_shape(1, E, H, F, dt, who)) return MOEP_EINVAL;
  if (dt != MOEP_BF16) return fail(MOEP_EUNSUPPORTED, "%s: packed weights exist for bf16 only", who);
  if (int st = check_alignment(H, F, dt, who)) return st;
  if (!W1 || !W3 || !W2 || !packed) return fail(MOEP_EINVAL, "%s: NULL pointer", who);
  if ((uintptr_t)packed & 255) return fail(MOEP_EINVAL, "%s: packed buffer must be 256-byte aligned", who);
  hipStream_t s = (hipStream_t)hip_stream;
  char* w13 = (char*)packed;
  char* w2 = w13 + (size_t)E * packed_b_bytes(F, H, true);
  if (int st = launch_pack_b_bf16(W1, W3, F, H, E, w13, s, "pack_w")) return st;
  return launch_pack_b_bf16(W2, nullptr, H, F, E, w2, s, "pack_w");
}

int moe_forward_pruned_skip_packed(const void* x, const void* Wgate, const void* packed_weights, int64_t T,
                                   int E, int H, int F, moep_dtype dt, int k, uint32_t kept_mask, float beta,
                                   void* out, uint8_t* skip_mask, float* logits_out, int32_t* top2_out,
                                   void* ws, size_t ws_bytes, void* hip_stream) {
  if (!packed_weights) return fail(MOEP_EINVAL, "moe_forward_pruned_skip_packed: packed_weights is NULL");
  return forward_pruned_skip(x, Wgate, nullptr, nullptr, nullptr, packed_weights, T, E, H, F, dt, k, kept_mask,
                             beta, out, skip_mask, logits_out, top2_out, ws, ws_bytes, hip_stream);
}


// ------------------------------------------------------------------ moe_forward_skip_topk
size_t moe_forward_skip_topk_workspace(int64_t T, int E, int H, int F, moep_dtype dt, int k) {
  if (!valid_shape(T, E, H, F, dt, "moe_forward_skip_topk_workspace")) return 0;
  if (k < 1 || k > 16) return 0;
  SkipPlan p;
  if (plan_skip(T, E, H, F, dt, k, &p)) return 0;
  return p.total;
}

int moe_forward_skip_topk(const void* x, const void* Wgate, const void* W1, const void* W3,
                          const void* W2, int64_t T, int E, int H, int F, moep_dtype dt, int k,
                          uint32_t kept_mask, float beta, void* out, int32_t* n_used,
                          float* logits_out, int32_t* topk_out, void* ws, size_t ws_bytes,
                          void* hip_stream) {
  const char* who = "moe_forward_skip_topk";
  if (!valid_shape(T, E, H, F, dt, who)) return MOEP_EINVAL;
  if (k < 1) return fail(MOEP_EINVAL, "%s: k=%d must be at least 1", who, k);
  if (k > 16) return fail(MOEP_EUNSUPPORTED, "%s: k=%d (at most 16 experts per token)", who, k);
  if (E < 32 && (kept_mask >> E)) return fail(MOEP_EINVAL, "%s: kept_mask 0x%x has bits beyond expert %d", who, kept_mask, E - 1);
  if (__builtin_popcount(kept_mask) < k) return fail(MOEP_EINVAL, "%s: kept_mask 0x%x keeps fewer than k=%d experts", who, kept_mask, k);
  if (!(beta >= 0.0f) || std::isinf(beta)) return fail(MOEP_EINVAL, "%s: beta must be finite and >= 0", who);
  if (int st = check_alignment(H, F, dt, who)) return st;
  if (!Wgate || !W1 || !W3 || !W2) return fail(MOEP_EINVAL, "%s: NULL weight pointer", who);
  if (T == 0) return MOEP_OK;
  if (!x || !out || !n_used) return fail(MOEP_EINVAL, "%s: NULL x, out or n_used", who);
  SkipPlan p;
  if (int st = plan_skip(T, E, H, F, dt, k, &p)) return st;
  if (int st = check_ws(ws, ws_bytes, p.total, who)) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  char* w = (char*)ws;
  float* logits = logits_out ? logits_out : (float*)(w + p.off_logits);
  if (int st = launch_router(x, Wgate, T, E, H, dt, logits, s)) return st;
  if (int st = launch_skip_topk_routing(p, logits, kept_mask, beta, n_used, topk_out, w, s)) return st;
  void* direct = dt == MOEP_BF16 ? out : nullptr;
  if (int st = run_routed_ffn(p, x, W1, W3, W2, dt, w, s, nullptr, nullptr, direct)) return st;
  return launch_skip_topk_combine(p, dt, out, w, s, direct != nullptr);
}

// ------------------------------------------------------------------ skip_calibrate_beta
size_t skip_calibrate_beta_workspace(int64_t T) {
  if (T < 1 || T >= ((int64_t)1 << 32)) return 0;
  return calibrate_workspace_bytes(T);
}

int skip_calibrate_beta(const float* logits, int64_t T, int E, uint32_t kept_mask, float* beta_out,
                        void* ws, size_t ws_bytes, void* hip_stream) {
  const char* who = "skip_calibrate_beta";
  if (T < 1 || T >= ((int64_t)1 << 32)) return fail(MOEP_EINVAL, "%s: T=%lld (the median needs at least one token)", who, (long long)T);
  if (E < 2 || E > 32) return fail(MOEP_EINVAL, "%s: E=%d out of range 2..32", who, E);
  if (E < 32 && (kept_mask >> E)) return fail(MOEP_EINVAL, "%s: kept_mask 0x%x has bits beyond expert %d", who, kept_mask, E - 1);
  if (__builtin_popcount(kept_mask) < 2) return fail(MOEP_EINVAL, "%s: kept_mask 0x%x keeps fewer than two experts", who, kept_mask);
  if (!logits || !beta_out) return fail(MOEP_EINVAL, "%s: NULL logits or beta_out", who);
  if (int st = check_ws(ws, ws_bytes, calibrate_workspace_bytes(T), who)) return st;
  return launch_calibrate_beta(logits, T, E, kept_mask, beta_out, (char*)ws, (hipStream_t)hip_stream);
}


// ------------------------------------------------------------------ expert_selection_stats
int expert_selection_stats(const float* logits, int64_t T, int E, int k, int r, int64_t* count,
                           int64_t* coselect, uint32_t* frequency_mask, void* hip_stream) {
  const char* who = "expert_selection_stats";
  if (T < 0) return fail(MOEP_EINVAL, "%s: T=%lld is negative", who, (long long)T);
  if (E < 1 || E > 32) return fail(MOEP_EINVAL, "%s: E=%d out of range 1..32", who, E);
  if (k < 1 || k > E) return fail(MOEP_EINVAL, "%s: k=%d out of range 1..E", who, k);
  if (!count || !coselect) return fail(MOEP_EINVAL, "%s: NULL count or coselect", who);
  if (T > 0 && !logits) return fail(MOEP_EINVAL, "%s: NULL logits", who);
  if (frequency_mask && (r < 1 || r > E)) return fail(MOEP_EINVAL, "%s: r=%d out of range 1..E", who, r);
  return launch_selection_stats(logits, T, E, k, r, count, coselect, frequency_mask, (hipStream_t)hip_stream);
}


// ------------------------------------------------------------------ rank-limited expert pass
size_t moe_expert_outputs_ranked_workspace(int64_t T, int E, int H, int F, moep_dtype dt, int n_rank) {
  if (!valid_shape(T, E, H, F, dt, "moe_expert_outputs_ranked_workspace")) return 0;
  if (n_rank < 1 || n_rank > 16 || n_rank > E) return 0;
  SkipPlan p;
  if (plan_skip(T, E, H, F, dt, n_rank, &p, false)) return 0;
  return p.total;
}

int moe_expert_outputs_ranked(const void* x, const void* Wgate, const void* W1, const void* W3,
                              const void* W2, int64_t T, int E, int H, int F, moep_dtype dt,
                              int n_rank, float* logits, int32_t* ranked_experts, int32_t* slot_of,
                              void* Yr, void* ws, size_t ws_bytes, void* hip_stream) {
  const char* who = "moe_expert_outputs_ranked";
  if (!valid_shape(T, E, H, F, dt, who)) return MOEP_EINVAL;
  if (n_rank < 1 || n_rank > E) return fail(MOEP_EINVAL, "%s: n_rank=%d out of range 1..E", who, n_rank);
  if (n_rank > 16) return fail(MOEP_EUNSUPPORTED, "%s: n_rank=%d (at most 16)", who, n_rank);
  if (int st = check_alignment(H, F, dt, who)) return st;
  if (!Wgate || !W1 || !W3 || !W2) return fail(MOEP_EINVAL, "%s: NULL weight pointer", who);
  if (T == 0) return MOEP_OK;
  if (!x || !logits || !ranked_experts || !slot_of || !Yr)
    return fail(MOEP_EINVAL, "%s: NULL x, logits, ranked_experts, slot_of or Yr", who);
  SkipPlan p;
  if (int st = plan_skip(T, E, H, F, dt, n_rank, &p, false)) return st;
  if (int st = check_ws(ws, ws_bytes, p.total, who)) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  char* w = (char*)ws;
  if (int st = launch_router(x, Wgate, T, E, H, dt, logits, s)) return st;
  const uint32_t all = E < 32 ? (1u << E) - 1u : 0xffffffffu;
  // beta = 0 keeps all n_rank experts of every token; the [T, n_rank] region of the workspace that would
  // hold the expert ids (they go to ranked_experts instead) takes the per-token counts.
  int32_t* n_used = (int32_t*)(w + p.off_pos) + (int64_t)n_rank * T;
  if (int st = launch_skip_topk_routing(p, logits, all, 0.0f, n_used, ranked_experts, w, s, slot_of)) return st;
  return run_routed_ffn(p, x, W1, W3, W2, dt, w, s, Yr);
}

int prune_enumerate_ranked(const float* logits, const int32_t* ranked_experts, const int32_t* slot_of,
                           const void* Yr, int64_t T, int E, int H, moep_dtype dt, int n_rank, int k,
                           int r, float* loss, int32_t* argmin, uint32_t* argmin_mask,
                           int64_t* unaffected_pairs, void* ws, size_t ws_bytes, void* hip_stream) {
  const char* who = "prune_enumerate_ranked";
  if (!valid_shape(T, E, H, 1, dt, who)) return MOEP_EINVAL;
  EnumPlan p;
  if (int st = plan_enumerate(T, E, H, k, r, &p)) return st;
  if (n_rank < p.n_act || n_rank > E || n_rank > 16)
    return fail(MOEP_EINVAL, "%s: n_rank=%d, but k=%d, r=%d can select any of a token's first %d ranked experts",
                who, n_rank, k, r, p.n_act);
  if (H % (dt == MOEP_BF16 ? 64 : 1))
    return fail(MOEP_EUNSUPPORTED, "%s: H=%d must be a multiple of 64 for bf16", who, H);
  if (!loss || !argmin || !argmin_mask) return fail(MOEP_EINVAL, "%s: NULL loss, argmin or argmin_mask", who);
  if (T > 0 && (!logits || !ranked_experts || !slot_of || !Yr))
    return fail(MOEP_EINVAL, "%s: NULL logits, ranked_experts, slot_of or Yr", who);
  if (int st = check_ws(ws, ws_bytes, p.total, who)) return st;
  RankedSource src{slot_of, ranked_experts, n_rank};
  return launch_enumerate(p, logits, Yr, dt, loss, argmin, argmin_mask, unaffected_pairs, (char*)ws,
                          (hipStream_t)hip_stream, &src);
}

}  // extern "C"
