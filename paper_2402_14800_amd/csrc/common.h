// Internal declarations shared by the host API and the kernel launchers of libmoeprune.
// Nothing here is part of the C ABI (that is include/moeprune.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "moeprune.h"

namespace moep {

// ---- errors -----------------------------------------------------------------
int fail(int status, const char* fmt, ...);   // records the thread's message, returns status

#define MOEP_HIP(expr)                                                                  \
  do {                                                                                  \
    hipError_t _e = (expr);                                                             \
    if (_e != hipSuccess)                                                               \
      return ::moep::fail(MOEP_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e));    \
  } while (0)

// ---- per-kernel timing ------------------------------------------------------
// A Timed object brackets the launches made during its lifetime with a pair of
// HIP events on `stream` when timing is enabled; otherwise it does nothing.
struct Timed {
  Timed(const char* kernel_name, hipStream_t stream);
  ~Timed();
  int slot;
  hipStream_t stream;
};

static inline size_t align256(size_t n) { return (n + 255) & ~size_t(255); }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t dtype_size(moep_dtype dt) { return dt == MOEP_BF16 ? 2 : 4; }

// ---- fp32 GEMM: C = epilogue(A B^T), A [M,K] and B [N,K] both K-contiguous, row-major operands -----
enum GemmEpilogue {
  EPI_STORE = 0,      // C[m,n] = acc                       (C in dt, N columns)
  EPI_SWIGLU = 1,     // C[m,n] = silu(A B0^T) * (A B1^T)    (C in dt, N columns)
  EPI_ROWSCALE_F32 = 2  // C[m,n] = row_scale[m] * acc        (C in fp32)
};

struct GemmArgs {
  const void* A = nullptr;       // [rows, K], leading dimension lda (elements)
  int64_t lda = 0;
  const int32_t* a_rows = nullptr;  // optional: logical row m reads A row a_rows[m]
  const void* B0 = nullptr;      // [N, K] (per expert), leading dimension K
  const void* B1 = nullptr;      // second weight for EPI_SWIGLU
  void* C = nullptr;             // [rows, N], leading dimension ldc (elements)
  int64_t ldc = 0;
  int64_t M = 0;                 // logical rows (dense mode) or upper bound on rows (grouped)
  int N = 0, K = 0;
  int epilogue = EPI_STORE;
  const float* row_scale = nullptr;
  // Grouped mode (rows partitioned into per-expert segments): tile t of the M
  // dimension covers rows [tile_row0[t], min(tile_row0[t] + BM, seg_end[tile_expert[t]]))
  // and multiplies with expert tile_expert[t]'s weights; tile_expert[t] < 0 = no work.
  const int32_t* tile_expert = nullptr;
  const int32_t* tile_row0 = nullptr;
  const int32_t* seg_end = nullptr;     // [E] end row (exclusive) of each expert's segment
  int64_t b_expert_stride = 0;          // elements between consecutive experts' weights
  int64_t max_m_tiles = 0;              // grouped: number of entries in tile_expert/tile_row0
  const int32_t* tiles_in_use = nullptr; // grouped, optional: device count of leading entries that hold work
};

constexpr int GEMM_BM = 256;   // rows per tile of either GEMM implementation's grouped map
// bf16 packed GEMM: M tiles per group of tiles that an XCD works through together, and output columns per tile,
// for the gate/up (SwiGLU) and the down projection (measured: the long-K down projection prefers 4 x 8 tiles per XCD)
constexpr int GEMM_GROUP_M_SWIGLU = 8, GEMM_GROUP_M_STORE = 4;
constexpr int GEMM_BN_SWIGLU = 128, GEMM_BN_STORE = 256;

int launch_gemm_f32(const GemmArgs& g, hipStream_t s, const char* name);

// ---- bf16 GEMM on packed operands (dense expert pass) ---------------------------------
// Operands are re-laid out once into 16 KB blocks of 256 rows x 32 k-values (the layout is described in
// gemm_bf16_packed.hip); EPI_SWIGLU writes its result as a packed A operand with K = N.
struct PackedGemmArgs {
  const void* A = nullptr;       // packed A operand, indexed by M tile
  const void* B = nullptr;       // packed_b_bytes(N, K, epilogue == EPI_SWIGLU) per expert
  void* C = nullptr;             // EPI_STORE / EPI_ROWSCALE_F32: row-major [rows, ldc]; EPI_SWIGLU: packed A operand, K = N
  int64_t ldc = 0;
  int64_t M = 0;                 // rows (dense mode)
  int N = 0, K = 0;
  int epilogue = EPI_STORE;
  const float* row_scale = nullptr;
  // Grouped mode: the same tile map as GemmArgs; A (and a packed C) hold one 256-row block per TILE.
  const int32_t* tile_expert = nullptr;
  const int32_t* tile_row0 = nullptr;
  const int32_t* seg_end = nullptr;
  const int32_t* tiles_in_use = nullptr;
  int64_t max_m_tiles = 0;
  // Grouped mode, optional: the order in which the launch walks its tiles, entry i = (M tile << 12) | N tile,
  // tiles_in_use x n_tiles entries (see order_kernel in skip.hip); without it groups of M tiles may straddle experts.
  const uint32_t* tile_order = nullptr;
  // Dense batched mode: `experts` GEMMs of the same shape in one launch; expert e reads A + e a_expert_bytes
  // (0: every expert reads the same A), B + e packed_b_bytes(..), and writes C + e c_expert_bytes.
  int experts = 1;
  int64_t a_expert_bytes = 0, c_expert_bytes = 0;
  // EPI_ROWSCALE_F32, optional: rows r with row_dest[r] >= 0 are not written to C but, rounded to bf16 and
  // unscaled (their scale is 1), to row row_dest[r] of `direct_out` (leading dimension ldc): the slots of
  // tokens that were routed to a single expert go straight to the layer output.
  const int32_t* row_dest = nullptr;
  void* direct_out = nullptr;
};
size_t packed_a_bytes(int64_t rows, int K);
size_t packed_b_bytes(int N, int K, bool gate_up_pair);
int launch_pack_a_bf16(const void* X, int64_t ld, int64_t rows, int K, void* dst, hipStream_t s, const char* name);
// grouped: block row p of tile t = row rows_of[tile_row0[t] + p] of X
int launch_pack_a_gathered_bf16(const void* X, int64_t ld, const int32_t* rows_of, const int32_t* tile_expert,
                                const int32_t* tile_row0, const int32_t* seg_end, const int32_t* tiles_in_use,
                                int64_t max_tiles, int K, void* dst, hipStream_t s, const char* name);
// W1 != nullptr: gate/up pair (blocks of 128 rows of W0 followed by the same 128 rows of W1); `experts`
// consecutive [N, K] matrices are packed into consecutive packed_b_bytes blocks
int launch_pack_b_bf16(const void* W0, const void* W1, int N, int K, int experts, void* dst, hipStream_t s,
                       const char* name);
int launch_gemm_bf16_packed(const PackedGemmArgs& g, hipStream_t s, const char* name);

// ---- router -------------------------------------------------------------------
int launch_router(const void* x, const void* Wgate, int64_t T, int E, int H, moep_dtype dt,
                  float* logits, hipStream_t s);
// bf16: the same logits (bit for bit) and the packed A-operand copy of x in one pass; MOEP_EUNSUPPORTED, with nothing
// launched and no message, for shapes without a fused kernel
int launch_router_and_pack_x(const void* x, const void* Wgate, int64_t T, int E, int H, float* logits, void* xpacked,
                             hipStream_t s);

// ---- enumeration ----------------------------------------------------------------
struct EnumPlan {
  int64_t T; int E, H, k, r;
  int kk;            // min(k, r): experts per token in the pruned layer
  int n_act;         // min(E, kk + E - r): rank positions that can be selected
  int64_t n_sub;     // C(E, r)
  int rec_floats;    // floats per token record
  int tok_tile;      // tokens per scoring block
  int64_t n_tok_tiles;
  bool use_lut;      // many subsets, few selections per token: score through per-token selection tables
  int n_combo;       // C(n_act, kk): selections per token
  int lut_spl;       // subsets per lane of the table scorer (0 without it)
  // workspace carving (byte offsets)
  size_t off_gram, off_rec, off_masks, off_partial, off_partial_cnt, off_qtab, off_sel, off_selbits, off_nib, total;
};
int plan_enumerate(int64_t T, int E, int H, int k, int r, EnumPlan* p);
// Expert outputs of the rank-limited pass: row slot_of[t, j] of Y is the output of expert
// experts[t, j], the token's j-th ranked expert, j < n_rank.
struct RankedSource {
  const int32_t* slot_of;
  const int32_t* experts;
  int n_rank;
};
int launch_enumerate(const EnumPlan& p, const float* logits, const void* Y, moep_dtype dt,
                     float* loss, int32_t* argmin, uint32_t* argmin_mask, int64_t* unaffected,
                     char* ws, hipStream_t s, const RankedSource* ranked = nullptr, bool reuse_gram = false);

// fp64 sum of n_tiles partial sums per subset (partial[tile * n_sub + subset]) in a fixed order -> loss; sum of the
// partial counts -> *unaffected (may be NULL); lowest-index argmin and its kept mask
int launch_reduce_argmin(const float* partial, const uint32_t* partial_cnt, int64_t n_tiles, int64_t n_sub, int E,
                         int r, float* loss, int32_t* argmin, uint32_t* argmin_mask, int64_t* unaffected,
                         hipStream_t s);
// masks[i] = kept mask of subset i
int launch_subset_masks(int E, int r, int64_t n_sub, uint32_t* masks, hipStream_t s);

// The same losses straight from the definition, without Gram matrices (enumerate_direct.hip).
struct DirectPlan {
  int64_t T; int E, H, k, r;
  int64_t n_sub;
  int blocks;        // workgroups, each walking tokens b, b + blocks, ...
  size_t lds_bytes;  // dynamic LDS per workgroup
  size_t off_masks, off_partial, off_partial_cnt, total;
};
int plan_enumerate_direct(int64_t T, int E, int H, int k, int r, moep_dtype dt, DirectPlan* p);
int launch_enumerate_direct(const DirectPlan& p, const float* logits, const void* Y, moep_dtype dt, float* loss,
                            int32_t* argmin, uint32_t* argmin_mask, int64_t* unaffected, char* ws, hipStream_t s);

// ---- skipping ---------------------------------------------------------------------
struct SkipPlan {
  int64_t T; int E, H, F;
  int ks;                // slots per token (2 for the top-2 rule, k for the generalised rule)
  int64_t max_slots;     // ks T
  int64_t max_tiles;     // upper bound on M tiles over all experts
  size_t off_logits, off_slot_token, off_slot_scale, off_slot_dest, off_pos, off_counts, off_seg_end,
         off_tile_expert, off_tile_row0, off_order_up, off_order_down, off_h, off_xp, off_w13, off_w2, off_slot_out, total;
  bool packed;           // bf16: packed-operand GEMMs (tile order tables are built)
};
int plan_skip(int64_t T, int E, int H, int F, moep_dtype dt, int ks, SkipPlan* p, bool with_slot_out = true);
int launch_skip_routing(const SkipPlan& p, const float* logits, uint32_t kept_mask, float beta, uint8_t* skip_mask,
                        int32_t* top2_out, char* ws, hipStream_t s);
// `singles_done`: tokens routed to a single expert already have their output (written by the down projection)
int launch_skip_combine(const SkipPlan& p, moep_dtype dt, const uint8_t* skip_mask, void* out,
                        char* ws, hipStream_t s, bool singles_done);
int launch_skip_topk_routing(const SkipPlan& p, const float* logits, uint32_t kept_mask, float beta,
                             int32_t* n_used, int32_t* topk_out, char* ws, hipStream_t s,
                             int32_t* pos_out = nullptr);
int launch_skip_topk_combine(const SkipPlan& p, moep_dtype dt, void* out, char* ws, hipStream_t s, bool singles_done);

// ---- beta calibration -----------------------------------------------------------------
size_t calibrate_workspace_bytes(int64_t T);
int launch_calibrate_beta(const float* logits, int64_t T, int E, uint32_t kept_mask, float* beta_out,
                          char* ws, hipStream_t s);

// ---- selection statistics ---------------------------------------------------------------
int launch_selection_stats(const float* logits, int64_t T, int E, int k, int r, int64_t* count, int64_t* co,
                           uint32_t* freq_mask, hipStream_t s);

// Host-side subset helpers (also used to fill the device mask table).
int64_t binomial(int n, int r);
uint32_t unrank_mask(int E, int r, int64_t idx);

}  // namespace moep
