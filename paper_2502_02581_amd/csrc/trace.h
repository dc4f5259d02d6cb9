// Development instrumentation of the GEMM kernels, compiled in only with -DMOE_TRACE (the library
// that ships is built without it: every macro below is then empty).  With it, the LDS-DMA core
// stamps the shader clock where a tile's phases end -- 0: entry, 1: first operand tiles in LDS (ring
// pipeline only), 2: K loop done, 3: epilogue done (first wavefront) -- and every tile of the GEMM
// kernels leaves one record {block, kernel id, group, column tile | kind << 8 | rows << 16, start,
// end, phase cycles}: times from the 100 MHz wall clock, phases (set-up and first loads, K loop,
// epilogue, rest) in shader-clock cycles.  moe_trace_read copies the records to the host.
#pragma once

#ifdef MOE_TRACE
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe {
__device__ long long g_ph[65536 * 4];
struct TraceRec {
  int32_t block, kernel, group, what;
  unsigned long long t0, t1;
  int32_t ph[4];
};
constexpr int kTraceMax = 1 << 18;
__device__ TraceRec g_trace[kTraceMax];
__device__ int g_trace_n;
__device__ __forceinline__ void trace_put(int kernel, int group, int what, unsigned long long t0) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const int i = atomicAdd(&g_trace_n, 1);
    if (i < kTraceMax) {
      TraceRec r = {(int32_t)(blockIdx.x + blockIdx.y * gridDim.x), kernel, group, what, t0, (unsigned long long)wall_clock64(), {0, 0, 0, 0}};
      const long long* ph = g_ph + (blockIdx.x & 0xffff) * 4;
      const long long now = clock64();
      r.ph[0] = (int32_t)(ph[1] - ph[0]); r.ph[1] = (int32_t)(ph[2] - ph[1]); r.ph[2] = (int32_t)(ph[3] - ph[2]);
      r.ph[3] = (int32_t)(now - ph[3]);
      g_trace[i] = r;
    }
  }
}
}  // namespace moe

#define MOE_PHASE(i) do { if (threadIdx.x == 0) moe::g_ph[(blockIdx.x & 0xffff) * 4 + (i)] = clock64(); } while (0)
#define MOE_TRACE_BEGIN()                                                        \
  const unsigned long long moe_trace_t0 = (unsigned long long)wall_clock64(); \
  const unsigned long long moe_trace_c0 = (unsigned long long)clock64();      \
  (void)moe_trace_c0
// row tiles: the group field carries the shader-clock cycles of the tile (shader clock = cycles / wall time)
#define MOE_TRACE_ROW_TILE(kernel, what) \
  moe::trace_put((kernel), (int)((unsigned long long)clock64() - moe_trace_c0), (what), moe_trace_t0)
#define MOE_TRACE_W_TILE(kernel, group, what) moe::trace_put((kernel), (group), (what), moe_trace_t0)
// copies the trace records to the host buffer (at most max_records), returns their number and clears the trace
#define MOE_TRACE_DEFINE_READER                                                                                       \
  extern "C" int moe_trace_read(void* host, int max_records) {                                                        \
    int n = 0;                                                                                                        \
    if (hipMemcpyFromSymbol(&n, HIP_SYMBOL(moe::g_trace_n), sizeof(int)) != hipSuccess) return -1;                   \
    if (n > moe::kTraceMax) n = moe::kTraceMax;                                                                       \
    if (n > max_records) n = max_records;                                                                             \
    if (n > 0 && hipMemcpyFromSymbol(host, HIP_SYMBOL(moe::g_trace), (size_t)n * sizeof(moe::TraceRec)) != hipSuccess) \
      return -1;                                                                                                      \
    int zero = 0;                                                                                                     \
    (void)hipMemcpyToSymbol(HIP_SYMBOL(moe::g_trace_n), &zero, sizeof(int));                                          \
    return n;                                                                                                         \
  }
#else
#define MOE_PHASE(i) do {} while (0)
#define MOE_TRACE_BEGIN() do {} while (0)
#define MOE_TRACE_ROW_TILE(kernel, what) do {} while (0)
#define MOE_TRACE_W_TILE(kernel, group, what) do {} while (0)
#define MOE_TRACE_DEFINE_READER
#endif
