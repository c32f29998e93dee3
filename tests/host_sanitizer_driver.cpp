// Host logic of libmoeprune under AddressSanitizer / UndefinedBehaviorSanitizer: subset rank / unrank, workspace
// planning and the argument-error paths of every entry point.  No kernel is launched and no GPU is needed: every
// call below either is pure host arithmetic or must be refused before it reaches the HIP runtime.
// Built and run by tests/test_host_sanitizers.py against the sanitized build of the library.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "moeprune.h"

static int failures = 0;
#define EXPECT(cond)                                                          \
  do {                                                                        \
    if (!(cond)) { ++failures; std::printf("FAILED line %d: %s\n", __LINE__, #cond); } \
  } while (0)

static int64_t binom(int n, int r) {
  if (r < 0 || r > n) return 0;
  int64_t c = 1;
  for (int i = 1; i <= r; ++i) c = c * (n - r + i) / i;
  return c;
}

int main() {
  // ---- subsets: every index of every (E, r) up to E = 14, plus the corners of E = 32
  for (int E = 1; E <= 14; ++E)
    for (int r = 1; r <= E; ++r) {
      const int64_t n = moep_num_subsets(E, r);
      EXPECT(n == binom(E, r));
      uint32_t prev = 0;
      for (int64_t i = 0; i < n; ++i) {
        uint32_t m = 0;
        EXPECT(moep_subset_unrank(E, r, i, &m) == MOEP_OK);
        EXPECT(__builtin_popcount(m) == r && (E == 32 || (m >> E) == 0));
        EXPECT(moep_subset_rank(E, r, m) == i);
        if (i > 0) {   // lexicographic order of the sorted tuples = descending order of the bit-reversed masks
          uint32_t a = __builtin_bitreverse32(prev), b = __builtin_bitreverse32(m);
          EXPECT(a > b);
        }
        prev = m;
      }
    }
  {
    uint32_t m = 0;
    EXPECT(moep_num_subsets(32, 16) == binom(32, 16));
    EXPECT(moep_subset_unrank(32, 16, moep_num_subsets(32, 16) - 1, &m) == MOEP_OK && m == 0xffff0000u);
    EXPECT(moep_subset_rank(32, 16, 0xffff0000u) == moep_num_subsets(32, 16) - 1);
    EXPECT(moep_subset_unrank(32, 32, 0, &m) == MOEP_OK && m == 0xffffffffu);
    EXPECT(moep_subset_unrank(32, 1, 31, &m) == MOEP_OK && m == 0x80000000u);
    EXPECT(moep_subset_unrank(8, 2, 28, &m) == MOEP_EINVAL && std::strlen(moep_last_error()) > 0);
    EXPECT(moep_subset_unrank(8, 2, -1, &m) == MOEP_EINVAL);
    EXPECT(moep_subset_unrank(8, 2, 0, nullptr) == MOEP_EINVAL);
    EXPECT(moep_num_subsets(0, 1) == -1 && moep_num_subsets(33, 2) == -1 && moep_num_subsets(8, 9) == -1);
    EXPECT(moep_subset_rank(8, 2, 0x7) == -1 && moep_subset_rank(8, 2, 0x101) == -1);
  }

  // ---- workspace planning over a grid of shapes, including the largest and degenerate ones
  const int64_t Ts[] = {0, 1, 255, 256, 257, 16384, 262144, (int64_t)1 << 30, -1, ((int64_t)1 << 30) + 1};
  const int Es[] = {0, 1, 2, 8, 16, 32, 33};
  for (int64_t T : Ts)
    for (int E : Es)
      for (moep_dtype dt : {MOEP_F32, MOEP_BF16}) {
        const size_t w1 = moe_expert_outputs_workspace(T, E, 4096, 14336, dt);
        const size_t w2 = moe_forward_skip_workspace(T, E, 4096, 14336, dt);
        const size_t w3 = moe_expert_outputs_packed_workspace(T, E, 4096, 14336, dt);
        const bool ok = T >= 0 && T <= ((int64_t)1 << 30) && E >= 1 && E <= 32;
        EXPECT(ok || (w1 == 0 && w2 == 0 && w3 == 0));
        for (int k : {1, 2, 4})
          for (int r = 0; r <= E + 1 && r <= 33; ++r) {
            const size_t we = prune_enumerate_workspace(T, E, 4096, k, r, dt);
            const bool ok_e = ok && k <= E && r >= 1 && r <= E && binom(E, r) <= ((int64_t)1 << 24);
            EXPECT(ok_e ? we >= 256 : we == 0);
          }
        for (int k : {0, 1, 4, 16, 17}) (void)moe_forward_skip_topk_workspace(T, E, 4096, 14336, dt, k);
        for (int n : {0, 1, 6, 16, 17}) (void)moe_expert_outputs_ranked_workspace(T, E, 4096, 14336, dt, n);
      }
  {
    const int rs[] = {6, 4, 8, 1};
    EXPECT(prune_enumerate_multi_workspace(262144, 8, 4096, 2, 4, rs, MOEP_BF16) >=
           prune_enumerate_workspace(262144, 8, 4096, 2, 4, MOEP_BF16));
    EXPECT(prune_enumerate_multi_workspace(262144, 8, 4096, 2, 0, rs, MOEP_BF16) == 0);
    EXPECT(prune_enumerate_multi_workspace(262144, 8, 4096, 2, 4, nullptr, MOEP_BF16) == 0);
    EXPECT(moe_packed_weights_bytes(8, 4096, 14336, MOEP_BF16) == (size_t)8 * 3 * 4096 * 14336 * 2);
    EXPECT(moe_packed_weights_bytes(8, 4096, 14336, MOEP_F32) == 0 && moe_packed_weights_bytes(8, 100, 64, MOEP_BF16) == 0);
    EXPECT(skip_calibrate_beta_workspace(0) == 0 && skip_calibrate_beta_workspace(1) > 0);
  }

  // ---- argument errors: every call must come back with a status and a message, having launched nothing
  void* p = (void*)(uintptr_t)(1 << 20);          // never dereferenced on the host
  float* fp = (float*)p;
  int32_t* ip = (int32_t*)p;
  uint32_t* up = (uint32_t*)p;
  EXPECT(moe_expert_outputs(p, p, p, p, p, 16, 0, 64, 64, MOEP_BF16, fp, p, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moe_expert_outputs(p, p, p, p, p, 16, 4, 60, 64, MOEP_BF16, fp, p, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(moe_expert_outputs(p, nullptr, p, p, p, 16, 4, 64, 64, MOEP_BF16, fp, p, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moe_expert_outputs(p, p, p, p, p, 16, 4, 64, 64, MOEP_BF16, fp, p, nullptr, 0, nullptr) == MOEP_EWORKSPACE);
  EXPECT(moe_expert_outputs(p, p, p, p, p, 16, 4, 64, 64, MOEP_BF16, fp, p, (char*)p + 8, (size_t)1 << 30, nullptr) == MOEP_EWORKSPACE);
  EXPECT(moe_expert_outputs(p, p, p, p, p, 16, 4, 64, 64, MOEP_BF16, fp, p, p, 16, nullptr) == MOEP_EWORKSPACE);
  EXPECT(moe_expert_outputs(p, p, p, p, p, 0, 4, 64, 64, MOEP_BF16, fp, p, nullptr, 0, nullptr) == MOEP_OK);   // empty batch
  EXPECT(moe_expert_outputs_packed(p, p, nullptr, 16, 4, 64, 64, MOEP_BF16, fp, p, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moe_expert_outputs_packed(p, p, p, 16, 4, 64, 64, MOEP_F32, fp, p, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(prune_enumerate(fp, p, 16, 8, 64, MOEP_BF16, 2, 9, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(prune_enumerate(fp, p, 16, 8, 64, MOEP_BF16, 0, 4, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(prune_enumerate(fp, p, 16, 32, 64, MOEP_BF16, 2, 16, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(prune_enumerate(fp, p, 16, 8, 100, MOEP_BF16, 2, 4, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(prune_enumerate(fp, p, 16, 8, 64, MOEP_BF16, 2, 4, nullptr, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(prune_enumerate(nullptr, p, 16, 8, 64, MOEP_BF16, 2, 4, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(prune_enumerate(fp, p, 16, 8, 64, MOEP_BF16, 2, 4, fp, ip, up, nullptr, p, 16, nullptr) == MOEP_EWORKSPACE);
  {
    const int rs[] = {6, 9};
    EXPECT(prune_enumerate_multi(fp, p, 16, 8, 64, MOEP_BF16, 2, 2, rs, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
    EXPECT(prune_enumerate_multi(fp, p, 16, 8, 64, MOEP_BF16, 2, 0, rs, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  }
  // Eq. 3 as written: its limits are argument errors, found before anything touches the GPU
  EXPECT(prune_enumerate_direct_workspace(262144, 8, 4096, 2, 4, MOEP_BF16) >= 512u * 70 * 8);
  EXPECT(prune_enumerate_direct_workspace(262144, 16, 2048, 4, 8, MOEP_BF16) == 0);            // 12870 subsets
  EXPECT(prune_enumerate_direct(fp, p, 16, 16, 64, MOEP_BF16, 4, 8, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(prune_enumerate_direct(fp, p, 16, 16, 64, MOEP_BF16, 5, 15, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(prune_enumerate_direct(fp, p, 16, 8, 16384, MOEP_BF16, 2, 6, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(prune_enumerate_direct(fp, p, 16, 8, 70, MOEP_F32, 2, 6, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(prune_enumerate_direct(fp, p, 16, 8, 64, MOEP_BF16, 2, 9, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(prune_enumerate_direct(fp, p, 16, 8, 64, MOEP_BF16, 2, 6, nullptr, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(prune_enumerate_direct(fp, nullptr, 16, 8, 64, MOEP_BF16, 2, 6, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(prune_enumerate_direct(fp, p, 16, 8, 64, MOEP_BF16, 2, 6, fp, ip, up, nullptr, p, 16, nullptr) == MOEP_EWORKSPACE);
  EXPECT(prune_enumerate_static(fp, p, 200000, 8, 64, MOEP_BF16, 2, 4, fp, ip, up, nullptr, nullptr) == MOEP_EWORKSPACE);
  EXPECT(prune_enumerate_static(fp, p, 100, 8, 64, MOEP_BF16, 2, 4, nullptr, ip, up, nullptr, nullptr) == MOEP_EINVAL);
  EXPECT(prune_enumerate_ranked(fp, ip, ip, p, 16, 8, 64, MOEP_BF16, 4, 2, 4, fp, ip, up, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  uint8_t* bp = (uint8_t*)p;
  EXPECT(moe_forward_skip(p, p, p, p, p, 16, 8, 64, 64, MOEP_BF16, 3, 0.5f, p, bp, nullptr, nullptr, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(moe_forward_skip(p, p, p, p, p, 16, 8, 64, 64, MOEP_BF16, 2, -1.0f, p, bp, nullptr, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moe_forward_skip(p, p, p, p, p, 16, 1, 64, 64, MOEP_BF16, 2, 0.5f, p, bp, nullptr, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moe_forward_pruned_skip(p, p, p, p, p, 16, 8, 64, 64, MOEP_BF16, 2, 0x100u, 0.5f, p, bp, nullptr, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moe_forward_pruned_skip(p, p, p, p, p, 16, 8, 64, 64, MOEP_BF16, 2, 0x1u, 0.5f, p, bp, nullptr, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moe_forward_pruned_skip_packed(p, p, nullptr, 16, 8, 64, 64, MOEP_BF16, 2, 0xffu, 0.5f, p, bp, nullptr, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moe_forward_skip_topk(p, p, p, p, p, 16, 8, 64, 64, MOEP_BF16, 17, 0xffu, 0.1f, p, ip, nullptr, nullptr, p, 1 << 20, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(moe_forward_skip_topk(p, p, p, p, p, 16, 8, 64, 64, MOEP_BF16, 4, 0x7u, 0.1f, p, ip, nullptr, nullptr, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moe_pack_weights(p, p, p, 8, 64, 64, MOEP_F32, p, nullptr) == MOEP_EUNSUPPORTED);
  EXPECT(moe_pack_weights(p, p, p, 8, 64, 64, MOEP_BF16, (char*)p + 16, nullptr) == MOEP_EINVAL);
  EXPECT(skip_calibrate_beta(fp, 0, 8, 0xffu, fp, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(skip_calibrate_beta(fp, 16, 8, 0x1u, fp, p, 1 << 20, nullptr) == MOEP_EINVAL);
  int64_t* lp = (int64_t*)p;
  EXPECT(expert_selection_stats(fp, 16, 8, 9, 4, lp, lp, up, nullptr) == MOEP_EINVAL);
  EXPECT(expert_selection_stats(fp, 16, 8, 2, 0, lp, lp, up, nullptr) == MOEP_EINVAL);
  EXPECT(moe_expert_outputs_ranked(p, p, p, p, p, 16, 8, 64, 64, MOEP_BF16, 9, fp, ip, ip, p, p, 1 << 20, nullptr) == MOEP_EINVAL);
  EXPECT(moep_mfma_ceiling(p, p, 1 << 20, 3, fp, 1 << 20, nullptr, nullptr) == MOEP_EINVAL);
  {
    const char* names[4]; double ms[4]; int64_t cnt[4]; float f[4];
    EXPECT(moep_timing_collect(nullptr, ms, cnt, 4) == -1);
    EXPECT(moep_timing_collect(names, ms, cnt, 4) == 0);       // nothing recorded
    EXPECT(moep_timing_records(names, f, 0) == -1);
    EXPECT(moep_timing_records(names, f, 4) == 0);
  }
  EXPECT(std::strlen(moep_last_error()) > 0);
  std::printf(failures ? "host sanitizer driver: %d check(s) failed\n" : "host sanitizer driver: all checks passed\n", failures);
  return failures ? 1 : 0;
}
