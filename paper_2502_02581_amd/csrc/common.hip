// Host-side error state and argument checks shared by all entry points.
#include <stdarg.h>
#include <string.h>

#include "moe_common.h"

namespace moe {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(const moe_shape_t* s, const char* who) {
  if (!s) {
    set_error("%s: shape is NULL", who);
    return MOE_EINVAL;
  }
  if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) {
    set_error("%s: unknown dtype %d", who, s->dtype);
    return MOE_EDTYPE;
  }
  if (s->gate != MOE_GATE_SOFTMAX && s->gate != MOE_GATE_SIGMOID) {
    set_error("%s: unknown gate %d", who, s->gate);
    return MOE_EDTYPE;
  }
  if (s->T < 0 || s->d <= 0 || s->d_ff <= 0 || s->E < 1 || s->E > MOE_MAX_EXPERTS || s->k < 1 ||
      s->k > s->E || s->k > MOE_MAX_TOPK) {
    set_error("%s: bad shape T=%d d=%d E=%d k=%d d_ff=%d", who, s->T, s->d, s->E, s->k, s->d_ff);
    return MOE_EINVAL;
  }
  if (s->d % 8 || s->d_ff % 8) {
    set_error("%s: d=%d and d_ff=%d must be multiples of 8", who, s->d, s->d_ff);
    return MOE_EINVAL;
  }
  if ((int64_t)s->T * s->k >= (int64_t)1 << 31 || (int64_t)s->T * s->k * s->d >= (int64_t)1 << 40) {
    set_error("%s: T*k=%lld overflows the index range", who, (long long)s->T * s->k);
    return MOE_EINVAL;
  }
  return MOE_OK;
}

int launch_status(const char* who) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("%s: launch failed: %s", who, hipGetErrorString(e));
    return MOE_ELAUNCH;
  }
  return MOE_OK;
}

}  // namespace moe

extern "C" int moe_abi_version(void) { return MOE_ABI_VERSION; }
extern "C" const char* moe_last_error(void) { return moe::g_err; }
