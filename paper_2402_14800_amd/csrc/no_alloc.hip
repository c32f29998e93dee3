// prune_enumerate_static: prune_enumerate for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  The Gram matrices, the per-token
// records and the partial sums of the scorer live in a fixed array in the library's own device data
// instead of a caller-supplied workspace; everything else (planning, kernels, launch order) is
// prune_enumerate's, so the outputs are the same bits.
#include <mutex>

#include "common.h"

namespace moep {
namespace {

// One copy per GPU that loads the library, held until the process ends.  In host code the array's name is a
// stand-in, not a device address: its address on the current device comes from hipGetSymbolAddress below and
// only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[MOEP_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
char* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device (looked up once per device, with that device current).
int scratch_on_current_device(char** out) {
  int dev = -1;
  MOEP_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices)
    return fail(MOEP_EUNSUPPORTED, "prune_enumerate_static: device ordinal %d beyond %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    MOEP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255))
      return fail(MOEP_EHIP, "prune_enumerate_static: bad address %p for the scratch array", p);
    g_scratch_ptr[dev] = (char*)p;
  }
  *out = g_scratch_ptr[dev];
  return MOEP_OK;
}

}  // namespace
}  // namespace moep

using namespace moep;

extern "C" int prune_enumerate_static(const float* logits, const void* Y, int64_t T, int E, int H, moep_dtype dt,
                                      int k, int r, float* loss, int32_t* argmin, uint32_t* argmin_mask,
                                      int64_t* unaffected_pairs, void* hip_stream) {
  const char* who = "prune_enumerate_static";
  if (dt != MOEP_F32 && dt != MOEP_BF16) return fail(MOEP_EINVAL, "%s: unknown dtype %d", who, (int)dt);
  if (T < 0 || T > (int64_t)1 << 30) return fail(MOEP_EINVAL, "%s: T=%lld out of range [0, 2^30]", who, (long long)T);
  if (E < 1 || E > 32) return fail(MOEP_EINVAL, "%s: E=%d out of range [1, 32]", who, E);
  if (H < 1) return fail(MOEP_EINVAL, "%s: H=%d must be positive", who, H);
  EnumPlan p;
  if (int st = plan_enumerate(T, E, H, k, r, &p)) return st;
  if (H % (dt == MOEP_BF16 ? 64 : 1))
    return fail(MOEP_EUNSUPPORTED, "%s: H=%d must be a multiple of 64 for bf16", who, H);
  if (!loss || !argmin || !argmin_mask) return fail(MOEP_EINVAL, "%s: NULL loss, argmin or argmin_mask", who);
  if (T > 0 && (!logits || !Y)) return fail(MOEP_EINVAL, "%s: NULL logits or Y", who);
  if (p.total > (size_t)MOEP_STATIC_SCRATCH_BYTES)
    return fail(MOEP_EWORKSPACE,
                "%s: T=%lld, E=%d, k=%d, r=%d needs %zu bytes of scratch, the built-in array holds %zu; "
                "use prune_enumerate with a workspace",
                who, (long long)T, E, k, r, p.total, (size_t)MOEP_STATIC_SCRATCH_BYTES);
  char* ws = nullptr;
  if (int st = scratch_on_current_device(&ws)) return st;
  // Nothing in the scratch has to start at zero: the Gram, record and partial-sum kernels write every
  // element that a later kernel of the same call reads.
  return launch_enumerate(p, logits, Y, dt, loss, argmin, argmin_mask, unaffected_pairs, ws,
                          (hipStream_t)hip_stream);
}
