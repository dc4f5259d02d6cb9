// Host-side error state and argument checks shared by all entry points.
#include <stdarg.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "moe_common.h"

namespace moe {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

#ifdef MOE_TUNE
int tune_knob(const char* name, int dflt) {
  const char* v = getenv(name);
  return v && *v ? atoi(v) : dflt;
}
#endif

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

// ---- profiling records -----------------------------------------------------------------------
struct ProfRec {
  const char* label;
  hipEvent_t start, stop;
};
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof;
static std::vector<hipEvent_t> g_event_pool;

bool profile_on() { return g_prof_on; }

static hipEvent_t take_event() {
  if (!g_event_pool.empty()) {
    hipEvent_t e = g_event_pool.back();
    g_event_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

void profile_push(const char* label, hipStream_t st, bool begin) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (begin) {
    ProfRec r = {label, take_event(), take_event()};
    (void)hipEventRecord(r.start, st);
    g_prof.push_back(r);
  } else {
    for (size_t i = g_prof.size(); i-- > 0;)
      if (g_prof[i].label == label) {
        (void)hipEventRecord(g_prof[i].stop, st);
        break;
      }
  }
}

}  // namespace moe

extern "C" int moe_profile_enable(int on) {
  using namespace moe;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  for (auto& r : g_prof) {
    g_event_pool.push_back(r.start);
    g_event_pool.push_back(r.stop);
  }
  g_prof.clear();
  g_prof_on = on != 0;
  return MOE_OK;
}

extern "C" size_t moe_profile_report(char* buf, size_t buf_bytes) {
  using namespace moe;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  struct Agg { std::string label; int n; double ms; };
  std::vector<Agg> agg;
  for (auto& r : g_prof) {
    if (hipEventSynchronize(r.stop) != hipSuccess) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) continue;
    size_t i = 0;
    for (; i < agg.size(); i++)
      if (agg[i].label == r.label) break;
    if (i == agg.size()) agg.push_back({r.label, 0, 0.0});
    agg[i].n++;
    agg[i].ms += ms;
  }
  std::string out;
  char line[160];
  for (auto& a : agg) {
    snprintf(line, sizeof(line), "%s %d %.6f\n", a.label.c_str(), a.n, a.ms);
    out += line;
  }
  if (buf && buf_bytes > 0) {
    size_t n = out.size() < buf_bytes - 1 ? out.size() : buf_bytes - 1;
    memcpy(buf, out.data(), n);
    buf[n] = 0;
  }
  return out.size() + 1;
}

namespace moe {
// plain 16-byte-per-lane copy; its known traffic calibrates the HBM counters of a profiler run
__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
}  // namespace moe

extern "C" int moe_copy_probe(const void* src, void* dst, size_t bytes, void* stream) {
  using namespace moe;
  if (!src || !dst || bytes == 0 || bytes % 16 || !aligned16(src) || !aligned16(dst)) {
    set_error("moe_copy_probe: needs two 16-byte aligned device buffers and a size that is a positive multiple of 16");
    return MOE_EINVAL;
  }
  const size_t n = bytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>((n + 255) / 256, 32768);
  {
    ProfScope prof("copy_probe_kernel", (hipStream_t)stream);
    hipLaunchKernelGGL(copy_probe_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, n);
  }
  return launch_status("moe_copy_probe");
}

namespace moe {
// Register-resident matrix loop: every wavefront issues `iters` rounds of 16 independent
// v_mfma_f32_32x32x16_bf16 on constant operands (16 accumulator tiles = all 256 accumulator registers,
// one wavefront per SIMD); no loads, no LDS.  What it sustains is the matrix pipe's rate at the clock
// the chip holds under that load.
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16_t;
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float* sink) {
  const int lane = threadIdx.x & 63;
  probe_bf16x8_t a, b;
#pragma unroll
  for (int i = 0; i < 8; i++) {
    a[i] = (__bf16)(0.001f * (float)((lane + i) % 7));
    b[i] = (__bf16)(0.002f * (float)((lane + 2 * i) % 5));
  }
  probe_f32x16_t acc[16];
#pragma unroll
  for (int j = 0; j < 16; j++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[j][r] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int j = 0; j < 16; j++) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 16; j++)
#pragma unroll
    for (int r = 0; r < 16; r++) s += acc[j][r];
  // keeps the loop alive; the sums are small positive numbers, so nothing is ever stored
  if (s == -1.f) sink[blockIdx.x * 256 + threadIdx.x] = s;
}
}  // namespace moe

extern "C" int moe_mfma_probe(int32_t n_blocks, int32_t iters, float* sink, double* flops_out, void* stream) {
  using namespace moe;
  if (n_blocks < 1 || n_blocks > (1 << 20) || iters < 1 || iters > (1 << 24) || !sink) {
    set_error("moe_mfma_probe: needs 1..2^20 blocks, 1..2^24 rounds and a device buffer of n_blocks * 256 floats");
    return MOE_EINVAL;
  }
  {
    ProfScope prof("mfma_probe_kernel", (hipStream_t)stream);
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)n_blocks), dim3(256), 0, (hipStream_t)stream, (int)iters, sink);
  }
  // 4 wavefronts x iters x 16 instructions x (2 * 32 * 32 * 16) FLOPs per block
  if (flops_out) *flops_out = (double)n_blocks * 4.0 * (double)iters * 16.0 * 32768.0;
  return launch_status("moe_mfma_probe");
}

extern "C" int moe_abi_version(void) { return MOE_ABI_VERSION; }
extern "C" const char* moe_last_error(void) { return moe::g_err; }
