/*
 * moeprune -- expert-subset scoring and dynamic skipping for one MoE layer on
 * AMD MI355X (gfx950).  C ABI; every kernel behind it is hand-written HIP.
 *
 * Notation follows the paper: n = E experts, k experts per token, r experts kept,
 * hidden size H, SwiGLU ffn size F, T tokens.
 *
 * Conventions shared by every entry point
 *   - All arrays are row-major and contiguous.  Pointers named below are DEVICE
 *     pointers unless a comment says "host".
 *   - Weights are stored out-features x in-features (y = x W^T).  W1 is the
 *     SiLU-gated branch, W3 the linear branch, W2 the down projection.
 *   - `dt` is the storage type of x, the weights, Y and out.  Router logits are
 *     always fp32.  bf16 operands are multiplied exactly and accumulated in fp32.
 *   - Ownership: the caller owns every buffer, including the workspace `ws`
 *     (size from the matching *_workspace query, 256-byte aligned).  The library
 *     allocates no device memory and keeps no pointer after the call returns.
 *   - All work is enqueued on `hip_stream` (a hipStream_t, NULL = the default
 *     stream) and the call returns without waiting for it; outputs are valid
 *     once the caller has synchronised the stream.
 *   - Only kernels are enqueued (no memset, no memcpy, no allocation), so a call can be captured
 *     into a HIP graph.  The first call that uses a GEMM kernel or the kernel of
 *     prune_enumerate_direct raises that kernel's dynamic LDS limit (hipFuncSetAttribute): make one
 *     eager call of an entry point before capturing it.
 *   - Return value: a moep_status.  Nothing throws or aborts across the ABI.
 *     After a non-zero status moep_last_error() describes it.  Inputs holding
 *     NaN or Inf give unspecified results.
 *   - Same inputs give bitwise identical outputs (no floating-point atomics).
 *   - State the library keeps.  Host: the calling thread's last error message; per GPU, behind a
 *     mutex, the compute-unit count and which kernels have had their LDS limit raised (so
 *     first calls from several host threads are safe); the event pool of moep_timing_*.  Device:
 *     512 bytes of 64-bit counters in the library's own device data, through which the persistent
 *     workgroups of the bf16 GEMM kernels line up (integer atomics on values that only grow and
 *     cannot wrap; timing depends on them, results never do), and the scratch array of
 *     prune_enumerate_static.  Calls that overlap in time on one GPU, on different streams, share
 *     the counters: workgroups of one call may then wait for those of the other, for a bounded time.
 *     The line-up takes workgroup b to run on XCD b % 8, as this part deals workgroups out; on a
 *     part that did otherwise it would cost time, never a result.
 *   - Entry points may be called from several host threads at once, each on its own stream and
 *     buffers (prune_enumerate_static excepted, see there).
 *   - Shape limits: 1 <= E <= 32; T >= 0 (T = 0 is a valid empty batch);
 *     for MOEP_BF16, H and F must be multiples of 64; for MOEP_F32, multiples of 4.
 *     x, the weights, Y and the other [.,H] arrays must be 16-byte aligned (MOEP_EUNSUPPORTED otherwise).
 */
#ifndef MOEPRUNE_H
#define MOEPRUNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOEP_OK = 0,
  MOEP_EINVAL = 1,       /* null pointer, size or parameter out of range      */
  MOEP_EUNSUPPORTED = 2, /* valid request this build has no kernel for        */
  MOEP_EWORKSPACE = 3,   /* workspace missing, misaligned or too small        */
  MOEP_EHIP = 4          /* a HIP runtime call or kernel launch failed        */
} moep_status;

typedef enum { MOEP_F32 = 0, MOEP_BF16 = 1 } moep_dtype;

/* ---- host-only helpers (no GPU needed) ------------------------------------ */

/* Number of kept-expert subsets, C(E,r) (Sec. 3.2).  -1 if E or r is out of range. */
int64_t moep_num_subsets(int E, int r);

/* Subset index <-> kept mask.  Subsets are indexed in lexicographic order of
 * their sorted expert-index tuples (index 0 keeps experts 0..r-1); bit e of the
 * mask is set iff expert e is kept.  `mask_out` is a host pointer.
 * unrank returns a moep_status; rank returns the index, or -1 if the mask does
 * not have exactly r bits below bit E. */
int moep_subset_unrank(int E, int r, int64_t idx, uint32_t* mask_out);
int64_t moep_subset_rank(int E, int r, uint32_t mask);

/* Message for the calling thread's last non-zero status (static storage, host). */
const char* moep_last_error(void);

/* ---- moe_expert_outputs ---------------------------------------------------- */
/* Sec. 3.1: router logits l = x Wgate^T and the SwiGLU output of EVERY expert on
 * EVERY token, Y[e,t,:] = (silu(x_t W1[e]^T) * (x_t W3[e]^T)) W2[e]^T -- the
 * quantities from which Eq. 2 and every pruned layer of Sec. 3.2 are formed.
 *   x [T,H], Wgate [E,H], W1 [E,F,H], W3 [E,F,H], W2 [E,H,F]   (dt)
 *   logits [T,E] fp32 (out), Y [E,T,H] dt (out)
 * The intermediate silu(.)*(.) is rounded to dt once, between the two GEMMs.
 * Workspace: MOEP_F32: one [T,F] matrix; MOEP_BF16: that matrix for as many experts as go into one
 * launch (all E of them up to 12 GiB, fewer beyond), a copy of x and a copy of every expert's
 * weights, all in the blocked operand layout of the GEMMs (rows padded to a multiple of 256). */
size_t moe_expert_outputs_workspace(int64_t T, int E, int H, int F, moep_dtype dt);
int moe_expert_outputs(const void* x, const void* Wgate, const void* W1, const void* W3,
                       const void* W2, int64_t T, int E, int H, int F, moep_dtype dt,
                       float* logits, void* Y, void* ws, size_t ws_bytes, void* hip_stream);

/* ---- prune_enumerate ------------------------------------------------------- */
/* Sec. 3.2, Eq. 3: for each of the C(E,r) kept sets C, route every token to its
 * top-min(k,r) experts among C (compare logits; ties to the lower index), weight
 * them by Eq. 1, and accumulate || F'(x,C) - F(x) ||^2 over all tokens and hidden
 * units, F(x) being Eq. 2 on the same logits and Y.
 *   logits [T,E] fp32, Y [E,T,H] dt
 *   loss [C(E,r)] fp32 (out): SQUARED Frobenius norm per subset, in subset-index order
 *   argmin [1] int32 (out): lowest index with the smallest loss
 *   argmin_mask [1] uint32 (out): its kept mask
 *   unaffected_pairs [1] int64 (out, may be NULL): number of (subset, token)
 *     pairs whose pruned routing equals the full routing (they contribute 0 exactly)
 * Computed through the per-token Gram matrix G_t = Y_t Y_t^T: with d = pruned
 * weights - full weights the error is d^T G_t d, the same real number as Eq. 3.
 * C(E,r) must not exceed 2^24.  T = 0 gives all-zero losses and argmin 0. */
size_t prune_enumerate_workspace(int64_t T, int E, int H, int k, int r, moep_dtype dt);
int prune_enumerate(const float* logits, const void* Y, int64_t T, int E, int H, moep_dtype dt,
                    int k, int r, float* loss, int32_t* argmin, uint32_t* argmin_mask,
                    int64_t* unaffected_pairs, void* ws, size_t ws_bytes, void* hip_stream);

/* The same for several r at once on the same logits and Y (e.g. the paper's r = 6 and r = 4): the
 * pass over Y that builds the per-token Gram matrices does not depend on r and runs once.
 *   rs [n_r] (host): the subset sizes, each 1 <= r <= E
 *   loss (out): the loss vectors one after the other, C(E, rs[0]) + C(E, rs[1]) + ... floats
 *   argmin, argmin_mask [n_r] (out), unaffected_pairs [n_r] (out, may be NULL): as above, per r
 * Each part is bit-identical to what prune_enumerate returns for that r. */
size_t prune_enumerate_multi_workspace(int64_t T, int E, int H, int k, int n_r, const int* rs,
                                       moep_dtype dt);
int prune_enumerate_multi(const float* logits, const void* Y, int64_t T, int E, int H, moep_dtype dt,
                          int k, int n_r, const int* rs, float* loss, int32_t* argmin,
                          uint32_t* argmin_mask, int64_t* unaffected_pairs, void* ws, size_t ws_bytes,
                          void* hip_stream);

/* ---- prune_enumerate_direct -------------------------------------------------- */
/* Sec. 3.2, Eq. 3 evaluated as it is written: arguments, outputs and conventions of prune_enumerate,
 * but F'(x_t, C) - F(x_t) = sum_e d_e E_e(x_t) is formed over the hidden units for every (subset,
 * token) pair whose routing changes (d = Eq. 1 weights of the pruned routing minus those of the full
 * routing, at most 2k experts) and its squares are summed; no Gram matrices.  Each token's E rows of Y
 * are read from memory once and kept in LDS while all subsets are scored, so the pass moves the bytes
 * of the Gram pass and does O(k H) arithmetic per pair instead of O(k^2).  Kept as the measured
 * alternative to the Gram path and as a cross-check on it with different arithmetic.
 *   - Limits (MOEP_EUNSUPPORTED beyond them): C(E,r) <= 128, k <= 4, H a multiple of 8 (bf16) or
 *     4 (fp32), E*H*sizeof(dt) + 11 KB within the 160 KB of LDS.
 *   - The losses agree with prune_enumerate's to fp32 rounding, not bit for bit. */
size_t prune_enumerate_direct_workspace(int64_t T, int E, int H, int k, int r, moep_dtype dt);
int prune_enumerate_direct(const float* logits, const void* Y, int64_t T, int E, int H, moep_dtype dt,
                           int k, int r, float* loss, int32_t* argmin, uint32_t* argmin_mask,
                           int64_t* unaffected_pairs, void* ws, size_t ws_bytes, void* hip_stream);

/* ---- prune_enumerate_static -------------------------------------------------- */
/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: prune_enumerate with no workspace argument.  The scratch
 * memory (Gram matrices, per-token records, partial sums) is a fixed array of
 * MOEP_STATIC_SCRATCH_BYTES in the library's own device data, one copy per GPU, held until the
 * process ends.  Arguments and outputs as prune_enumerate, bit for bit.
 *   - Limit: prune_enumerate_workspace(T, E, H, k, r, dt) must not exceed MOEP_STATIC_SCRATCH_BYTES
 *     (e.g. E = 8, r = 4: about 70000 tokens; E = 16, r = 8: about 5000); beyond it the call returns
 *     MOEP_EWORKSPACE and launches nothing.
 *   - The call allocates and frees nothing and enqueues kernels only.  The first call on a GPU looks
 *     the array's address up (hipGetSymbolAddress): make it outside graph capture.
 *   - Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race and give undefined losses.  Calls one after the other on a
 *     stream are independent: nothing is carried over from the previous call. */
#define MOEP_STATIC_SCRATCH_BYTES (32u << 20)
int prune_enumerate_static(const float* logits, const void* Y, int64_t T, int E, int H, moep_dtype dt,
                           int k, int r, float* loss, int32_t* argmin, uint32_t* argmin_mask,
                           int64_t* unaffected_pairs, void* hip_stream);

/* ---- rank-limited expert pass ---------------------------------------------- */
/* A layer pruned to r experts routes a token to the first min(k,r) KEPT experts of its ranking
 * (Sec. 3.2); at most E - r experts are missing, so only the token's first
 * n_act = min(E, min(k,r) + E - r) ranked experts can ever be selected by any of the C(E,r)
 * pruned layers (or by the full layer).  moe_expert_outputs_ranked therefore runs each token
 * through its n_rank best-ranked experts only -- n_rank / E of the FLOPs of moe_expert_outputs --
 * and prune_enumerate_ranked scores the subsets from those outputs; the losses are the same real
 * numbers as prune_enumerate's whenever n_rank >= n_act.
 *   n_rank: 1 .. min(E, 16)
 *   logits [T,E] fp32 (out)
 *   ranked_experts [T,n_rank] int32 (out): the token's experts by descending logit, ties to the lower index
 *   slot_of [T,n_rank] int32 (out): row of Yr holding the output of ranked_experts[t,j] on token t
 *   Yr [T*n_rank, H] dt (out): expert outputs, rows grouped by expert, ascending token within an expert;
 *     row slot_of[t,j] is bit-identical to Y[ranked_experts[t,j], t, :] of moe_expert_outputs
 * prune_enumerate_ranked: arguments as prune_enumerate, with (ranked_experts, slot_of, Yr, n_rank)
 * in place of Y; n_rank < n_act(k, r) is MOEP_EINVAL.  Workspace: prune_enumerate_workspace. */
size_t moe_expert_outputs_ranked_workspace(int64_t T, int E, int H, int F, moep_dtype dt, int n_rank);
int moe_expert_outputs_ranked(const void* x, const void* Wgate, const void* W1, const void* W3,
                              const void* W2, int64_t T, int E, int H, int F, moep_dtype dt,
                              int n_rank, float* logits, int32_t* ranked_experts, int32_t* slot_of,
                              void* Yr, void* ws, size_t ws_bytes, void* hip_stream);
int prune_enumerate_ranked(const float* logits, const int32_t* ranked_experts, const int32_t* slot_of,
                           const void* Yr, int64_t T, int E, int H, moep_dtype dt, int n_rank, int k,
                           int r, float* loss, int32_t* argmin, uint32_t* argmin_mask,
                           int64_t* unaffected_pairs, void* ws, size_t ws_bytes, void* hip_stream);

/* ---- moe_forward_skip ------------------------------------------------------ */
/* Sec. 3.3 with the output of App. A.2, k = 2: per token take the top-2 experts
 * e0, e1; skip e1 iff w_e1 < beta * w_e0, decided as (l_e1 - l_e0) < ln(beta) in
 * fp32 (beta = 0 never skips); out = E_e0(x) for skipped tokens, else Eq. 2.
 * Only routed (token, expert) pairs are pushed through an expert.
 *   x, Wgate, W1, W3, W2 as above; beta >= 0
 *   out [T,H] dt (out), skip_mask [T] uint8 (out, 1 = second expert skipped)
 *   logits_out [T,E] fp32 (out, may be NULL): the router logits used, bit-identical
 *     to those moe_expert_outputs returns for the same x and Wgate
 *   top2_out [T,2] int32 (out, may be NULL): e0, e1 per token
 * k must be 2 (MOEP_EUNSUPPORTED otherwise). */
size_t moe_forward_skip_workspace(int64_t T, int E, int H, int F, moep_dtype dt);
int moe_forward_skip(const void* x, const void* Wgate, const void* W1, const void* W3,
                     const void* W2, int64_t T, int E, int H, int F, moep_dtype dt, int k,
                     float beta, void* out, uint8_t* skip_mask, float* logits_out,
                     int32_t* top2_out, void* ws, size_t ws_bytes, void* hip_stream);

/* ---- moe_forward_pruned_skip ---------------------------------------------- */
/* The deployable layer after pruning (Sec. 3.2: the experts outside the kept set C and their
 * routing weights are removed), optionally with dynamic skipping on top (Sec. 3.3: the two can be
 * used together).  Exactly moe_forward_skip, except that the top-2 experts are taken among the
 * experts whose bit is set in `kept_mask` (bit e = expert e; at least two bits below bit E).
 * With beta = 0 the output is F'(x, C) of Sec. 3.2; with every bit set it is moe_forward_skip.
 * Weights and logits keep their original expert indexing; removed experts are simply never
 * routed to.  Workspace: moe_forward_skip_workspace. */
int moe_forward_pruned_skip(const void* x, const void* Wgate, const void* W1, const void* W3,
                            const void* W2, int64_t T, int E, int H, int F, moep_dtype dt, int k,
                            uint32_t kept_mask, float beta, void* out, uint8_t* skip_mask,
                            float* logits_out, int32_t* top2_out, void* ws, size_t ws_bytes,
                            void* hip_stream);

/* ---- packed expert weights (serving loops) ----------------------------------- */
/* The bf16 expert GEMMs read their operands in a blocked layout; the forward calls above re-lay
 * the layer's expert weights out on every call (a read and a write of all of them).  A caller
 * that runs the same layer many times (token generation with dynamic skipping, Sec. 3.3 and the
 * speed-up table of Sec. 4) does it once:
 *   moe_packed_weights_bytes: size of the packed copy of W1, W3, W2 (0 if dt is not MOEP_BF16 or
 *     H, F are not multiples of 64);
 *   moe_pack_weights: W1, W3 [E,F,H], W2 [E,H,F] -> packed (device, caller-owned, 256-byte
 *     aligned, moe_packed_weights_bytes bytes); asynchronous on hip_stream;
 *   moe_forward_pruned_skip_packed: moe_forward_pruned_skip with `packed_weights` in place of
 *     W1, W3, W2; same outputs bit for bit, same workspace (moe_forward_skip_workspace).
 *   moe_expert_outputs_packed: moe_expert_outputs with `packed_weights` in place of W1, W3, W2 (a
 *     calibration loop that pushes batch after batch through the same layer, Sec. 3.2); same outputs
 *     bit for bit; workspace moe_expert_outputs_packed_workspace (no room for weights).
 * MOEP_EUNSUPPORTED for MOEP_F32 (fp32 storage has no packed form). */
size_t moe_packed_weights_bytes(int E, int H, int F, moep_dtype dt);
int moe_pack_weights(const void* W1, const void* W3, const void* W2, int E, int H, int F,
                     moep_dtype dt, void* packed, void* hip_stream);
size_t moe_expert_outputs_packed_workspace(int64_t T, int E, int H, int F, moep_dtype dt);
int moe_expert_outputs_packed(const void* x, const void* Wgate, const void* packed_weights, int64_t T,
                              int E, int H, int F, moep_dtype dt, float* logits, void* Y, void* ws,
                              size_t ws_bytes, void* hip_stream);
int moe_forward_pruned_skip_packed(const void* x, const void* Wgate, const void* packed_weights,
                                   int64_t T, int E, int H, int F, moep_dtype dt, int k,
                                   uint32_t kept_mask, float beta, void* out, uint8_t* skip_mask,
                                   float* logits_out, int32_t* top2_out, void* ws, size_t ws_bytes,
                                   void* hip_stream);

/* ---- moe_forward_skip_topk -------------------------------------------------- */
/* Dynamic skipping for top-k routing, 1 <= k <= 16 (appendix on the theory of dynamic skipping).
 * Per token, with w_1 >= ... >= w_k the Eq. 1 weights of its top-k experts among `kept_mask`
 * (ties to the lower index), the top-i* experts stay, where
 *     i* = min { i in 1..k : sum_{m>i} w_m <= beta * sum_{m<=k} w_m },
 * and out = sum_{m<=i*} w_m E_m(x) / sum_{m<=i*} w_m.  beta = 0 keeps all k (Eq. 2), beta >= 1
 * keeps only the best expert.  For k = 2 this is the rule of moe_forward_skip with its beta set
 * to b / (1 - b) (up to "<" against "<=").  The decision is taken in fp64 on the fp32 logits.
 *   x, weights, out, logits_out as in moe_forward_skip
 *   n_used [T] int32 (out): i* per token
 *   topk_out [T,k] int32 (out, may be NULL): the top-k experts, best first
 * Workspace: moe_forward_skip_topk_workspace (grows with k). */
size_t moe_forward_skip_topk_workspace(int64_t T, int E, int H, int F, moep_dtype dt, int k);
int moe_forward_skip_topk(const void* x, const void* Wgate, const void* W1, const void* W3,
                          const void* W2, int64_t T, int E, int H, int F, moep_dtype dt, int k,
                          uint32_t kept_mask, float beta, void* out, int32_t* n_used,
                          float* logits_out, int32_t* topk_out, void* ws, size_t ws_bytes,
                          void* hip_stream);

/* ---- skip_calibrate_beta ---------------------------------------------------- */
/* The threshold of Sec. 3.3 as the paper sets it (Sec. 3.3; appendix on experiment details):
 * the median over the T calibration tokens of w_e1 / w_e0 = exp(l_e1 - l_e0), e0 and e1 the
 * token's top-2 experts among `kept_mask`.  For even T the mean of the two middle values.  The
 * order statistics are selected exactly on the fp32 differences l_e1 - l_e0.
 *   logits [T,E] fp32, T >= 1;  beta_out [1] fp32 (DEVICE, out)
 * Passing the result to moe_forward_skip on the same tokens skips half of them (within 1/T
 * when no two tokens share the same difference). */
size_t skip_calibrate_beta_workspace(int64_t T);
int skip_calibrate_beta(const float* logits, int64_t T, int E, uint32_t kept_mask, float* beta_out,
                        void* ws, size_t ws_bytes, void* hip_stream);

/* ---- expert_selection_stats -------------------------------------------------- */
/* Selection statistics of a calibration set, and the activation-frequency baseline built on them
 * (Sec. 4.1, comparison with other expert pruning baselines; appendix on expert selection tendency).
 *   logits [T,E] fp32; top-k by logit, ties to the lower index, 1 <= k <= E
 *   count [E] int64 (out): tokens whose top-k contains expert e
 *   coselect [E,E] int64 (out): tokens whose top-k contains both i and j (diagonal = count)
 *   frequency_mask [1] uint32 (out, may be NULL): kept mask of the baseline that discards the
 *     E - r least selected experts (on equal counts the lower index is kept); r is ignored if NULL
 * Outputs are overwritten, not accumulated.  T = 0 gives zeros. */
int expert_selection_stats(const float* logits, int64_t T, int E, int k, int r, int64_t* count,
                           int64_t* coselect, uint32_t* frequency_mask, void* hip_stream);

/* ---- per-kernel timing (for benchmarks) ------------------------------------ */
/* While enabled, every kernel launch is bracketed by HIP events on its stream.
 * moep_timing_collect waits for the recorded events, adds them up per kernel and
 * clears the record; `names`/`total_ms`/`launches` are host arrays of `cap`
 * entries (names: static strings).  Returns the number of kernels seen, or -1.
 * At most 8192 launches are recorded between collects; later ones go untimed. */
int moep_timing_enable(int on);
int moep_timing_collect(const char** names, double* total_ms, int64_t* launches, int cap);
/* The same record launch by launch, in launch order (for medians and minima): names[i], ms[i] for
 * up to `cap` launches; returns how many were written, or -1.  Clears the record like collect. */
int moep_timing_records(const char** names, float* ms, int cap);

/* An empirical ceiling for the bf16 GEMM kernels (for benchmarks): one launch of the MFMA stream of
 * their K loop and nothing else -- same launch shape, instruction, accumulator tiling and order, no
 * LDS, memory or barrier traffic -- `steps` K steps (even) per wavefront.  The operand registers are
 * filled from `a_src` and `b_src` (DEVICE, bf16 data such as the layer's x and W1; 65536 bytes per
 * compute unit are read from each, `src_bytes` says how many each holds), because the clock this
 * part sustains depends on the operand bits.  `sink` (DEVICE, 256 floats per compute unit, count in
 * `sink_floats`) receives sums nobody needs.  `flop_out` (host, may be NULL) receives the floating-
 * point operations of the launch; time it with moep_timing_* (kernel name "mfma_ceiling"). */
int moep_mfma_ceiling(const void* a_src, const void* b_src, size_t src_bytes, int steps, float* sink,
                      size_t sink_floats, double* flop_out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MOEPRUNE_H */
