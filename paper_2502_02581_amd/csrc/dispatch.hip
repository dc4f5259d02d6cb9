// moe_dispatch: stable counting sort of the T*k assignments by expert, then the row copy.
//
//   1. dispatch_count  one wavefront per chunk of kChunk assignments: LDS histogram over experts
//                      (LDS atomics are used for the COUNTS only, so the result does not depend
//                      on their order), written to ws as hist[chunk][e].
//   2. dispatch_scan   one block: exclusive scan over chunks per expert (in place), counts,
//                      and the exclusive scan over experts (offsets).
//   3. dispatch_rank   one wavefront per chunk: walks its chunk in assignment order; the rank of
//                      an assignment among equal experts inside a 64-wide step comes from
//                      ballots in lane order, so row_of is the same on every run (stable sort).
//   4. dispatch_rows   one block per token: reads the token row once, writes it to its k rows.
#include <mutex>

#include "moe_common.h"

namespace moe {

constexpr int kChunk = 256;  // assignments per wavefront in steps 1 and 3

__global__ __launch_bounds__(64) void dispatch_count(const int32_t* __restrict__ topk_idx, int A, int E,
                                                     int32_t* __restrict__ hist) {
  __shared__ int32_t cnt[MOE_MAX_EXPERTS];
  const int lane = threadIdx.x;
  const int chunk = blockIdx.x;
  for (int e = lane; e < E; e += 64) cnt[e] = 0;
  __syncthreads();
  const int a0 = chunk * kChunk;
  for (int s = 0; s < kChunk; s += 64) {
    int a = a0 + s + lane;
    if (a < A) {
      int e = topk_idx[a];
      if (e >= 0 && e < E) atomicAdd(&cnt[e], 1);
    }
  }
  __syncthreads();
  for (int e = lane; e < E; e += 64) hist[(size_t)chunk * E + e] = cnt[e];
}

// The chunks are cut into C equal runs (C = 1024 / E rounded down to a power of two) so that all 1024
// threads work: thread (c, e) first sums run c of expert e, the run sums are scanned over c, then
// the thread rewrites its run as exclusive prefixes.  Loads go eight at a time ahead of the
// dependent additions and stores.
__global__ __launch_bounds__(1024) void dispatch_scan(int32_t* __restrict__ hist, int n_chunks, int E,
                                                      int32_t* __restrict__ counts,
                                                      int32_t* __restrict__ offsets) {
  __shared__ int32_t sc[MOE_MAX_EXPERTS];
  __shared__ int32_t part[1024];
  int C = 1;
  while (C * 2 * E <= 1024) C *= 2;
  const int c = threadIdx.x / E, e_run = threadIdx.x - c * E;
  const int per = (n_chunks + C - 1) / C;
  const int w0 = min(n_chunks, c * per), w1 = min(n_chunks, w0 + per);
  const bool worker = c < C;
  if (worker) {
    int sum = 0;
    for (int w = w0; w < w1; w += 8) {
      int v[8];
#pragma unroll
      for (int q = 0; q < 8; q++) v[q] = w + q < w1 ? hist[(size_t)(w + q) * E + e_run] : 0;
#pragma unroll
      for (int q = 0; q < 8; q++) sum += v[q];
    }
    part[c * E + e_run] = sum;
  }
  __syncthreads();
  if (worker) {
    int run = 0;
    for (int q = 0; q < c; q++) run += part[q * E + e_run];
    for (int w = w0; w < w1; w += 8) {
      int v[8];
#pragma unroll
      for (int q = 0; q < 8; q++) v[q] = w + q < w1 ? hist[(size_t)(w + q) * E + e_run] : 0;
#pragma unroll
      for (int q = 0; q < 8; q++) {
        if (w + q < w1) hist[(size_t)(w + q) * E + e_run] = run;
        run += v[q];
      }
    }
  }
  const int e = threadIdx.x;
  int run = 0;
  if (e < E) {
    for (int q = 0; q < C; q++) run += part[q * E + e];
    counts[e] = run;
  }
  sc[e] = e < E ? run : 0;
  __syncthreads();
  // inclusive Hillis-Steele scan over the (at most 1024) experts
  for (int step = 1; step < MOE_MAX_EXPERTS; step <<= 1) {
    int add = e >= step ? sc[e - step] : 0;
    __syncthreads();
    sc[e] += add;
    __syncthreads();
  }
  if (e < E) offsets[e + 1] = sc[e];
  if (e == 0) offsets[0] = 0;
}

__global__ __launch_bounds__(64) void dispatch_rank(const int32_t* __restrict__ topk_idx, int A, int E,
                                                    const int32_t* __restrict__ hist,
                                                    const int32_t* __restrict__ offsets,
                                                    int32_t* __restrict__ row_of,
                                                    int32_t* __restrict__ src_of) {
  __shared__ int32_t nxt[MOE_MAX_EXPERTS];
  const int lane = threadIdx.x;
  const int chunk = blockIdx.x;
  for (int e = lane; e < E; e += 64) nxt[e] = offsets[e] + hist[(size_t)chunk * E + e];
  __syncthreads();
  const int a0 = chunk * kChunk;
  const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  for (int s = 0; s < kChunk; s += 64) {
    const int a = a0 + s + lane;
    int e = -1;
    if (a < A) {
      e = topk_idx[a];
      if (e < 0 || e >= E) e = -1;
    }
    const bool valid = e >= 0;
    uint64_t todo = __ballot(valid);
    int rank = 0, group = 0;
    bool last = false;
    while (todo) {
      int leader = __ffsll((unsigned long long)todo) - 1;
      int le = __shfl(e, leader, kWave);
      uint64_t same = __ballot(valid && e == le);
      if (valid && e == le) {
        rank = __popcll(same & lt_mask);
        group = __popcll(same);
        last = (same >> lane) == 1ull;  // highest lane of the group
      }
      todo &= ~same;
    }
    int r = 0;
    if (valid) r = nxt[e] + rank;
    __syncthreads();
    if (valid && last) nxt[e] += group;
    __syncthreads();
    if (valid) {
      row_of[a] = r;
      src_of[r] = a;
    }
  }
}

// Xp[row_of[t*k+j], :] = X[t, :], 16 bytes per lane per access.  K > 0: k known at compile time.
template <int K>
__global__ __launch_bounds__(256) void dispatch_rows(const uint4* __restrict__ X,
                                                     const int32_t* __restrict__ row_of, int k_rt,
                                                     int vec_per_row, uint4* __restrict__ Xp) {
  constexpr int KM = K > 0 ? K : 1;
  const int k = K > 0 ? K : k_rt;
  const int t = blockIdx.x;
  const uint4* src = X + (size_t)t * vec_per_row;
  if (K > 0) {
    uint4* dst[KM];
#pragma unroll
    for (int j = 0; j < KM; j++) dst[j] = Xp + (size_t)row_of[(size_t)t * k + j] * vec_per_row;
    // two pieces per thread and trip: both loads are issued before the 2k stores
    int c = threadIdx.x;
    for (; c + (int)blockDim.x < vec_per_row; c += 2 * blockDim.x) {
      const uint4 v0 = src[c], v1 = src[c + blockDim.x];
#pragma unroll
      for (int j = 0; j < KM; j++) {
        dst[j][c] = v0;
        dst[j][c + blockDim.x] = v1;
      }
    }
    if (c < vec_per_row) {
      const uint4 v0 = src[c];
#pragma unroll
      for (int j = 0; j < KM; j++) dst[j][c] = v0;
    }
  } else {
    for (int c = threadIdx.x; c < vec_per_row; c += blockDim.x) {
      uint4 v = src[c];
      for (int j = 0; j < k; j++) {
        int r = row_of[(size_t)t * k + j];
        Xp[(size_t)r * vec_per_row + c] = v;
      }
    }
  }
}

}  // namespace moe

namespace moe {
// the four launches of a dispatch; `hist` is scratch of n_chunks * E counters (every one is written
// by dispatch_count before anything reads it)
static void dispatch_launch(const moe_shape_t* shape, const void* X, const int32_t* topk_idx, int32_t* counts,
                            int32_t* offsets, int32_t* row_of, int32_t* src_of, void* Xp, int32_t* hist,
                            hipStream_t st) {
  const int A = shape->T * shape->k;
  const int n_chunks = (A + kChunk - 1) / kChunk;
  if (n_chunks > 0) {
    ProfScope prof("dispatch_count", st);
    hipLaunchKernelGGL(dispatch_count, dim3(n_chunks), dim3(64), 0, st, topk_idx, A, shape->E, hist);
  }
  {
    ProfScope prof("dispatch_scan", st);
    hipLaunchKernelGGL(dispatch_scan, dim3(1), dim3(1024), 0, st, hist, n_chunks, shape->E, counts, offsets);
  }
  if (n_chunks > 0) {
    {
      ProfScope prof("dispatch_rank", st);
      hipLaunchKernelGGL(dispatch_rank, dim3(n_chunks), dim3(64), 0, st, topk_idx, A, shape->E, hist, offsets,
                         row_of, src_of);
    }
    ProfScope prof("dispatch_rows", st);
    const int vec_per_row = (int)((size_t)shape->d * elem_size(shape->dtype) / 16);
#define MOE_ROWS(K)                                                                                       \
  hipLaunchKernelGGL(dispatch_rows<K>, dim3(shape->T), dim3(256), 0, st, (const uint4*)X, row_of, shape->k, \
                     vec_per_row, (uint4*)Xp)
    switch (shape->k) {
      case 1: MOE_ROWS(1); break;
      case 2: MOE_ROWS(2); break;
      case 4: MOE_ROWS(4); break;
      case 8: MOE_ROWS(8); break;
      default: MOE_ROWS(0); break;
    }
#undef MOE_ROWS
  }
}

// Scratch of moe_dispatch_static: one array per GPU, part of the loaded code object, so that no call
// allocates.  Host code must not use the symbol's name as an address: the per-device address comes
// from hipGetSymbolAddress, once per device, and is what the kernels receive.
constexpr size_t kStaticHistInts = (size_t)MOE_DISPATCH_STATIC_MAX_COUNTERS;
static __device__ __align__(256) int32_t scratch[kStaticHistInts];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static int32_t* g_scratch_ptr[kMaxDevices];  // per device, set on the first call with that device current

// address of the current device's scratch array, or NULL with the error text set
static int32_t* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_error("moe_dispatch_static: no current device (or a device index above %d)", kMaxDevices - 1);
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      set_error("moe_dispatch_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = (int32_t*)p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace moe

extern "C" size_t moe_dispatch_workspace_bytes(const moe_shape_t* shape) {
  using namespace moe;
  if (!shape || shape->E < 1 || shape->T < 0 || shape->k < 1) return 0;
  size_t A = (size_t)shape->T * shape->k;
  size_t n_chunks = (A + kChunk - 1) / kChunk;
  return align_up((n_chunks > 0 ? n_chunks : 1) * (size_t)shape->E * sizeof(int32_t), 256);
}

extern "C" int moe_dispatch(const moe_shape_t* shape, const void* X, const int32_t* topk_idx, int32_t* counts,
                            int32_t* offsets, int32_t* row_of, int32_t* src_of, void* Xp, void* ws,
                            size_t ws_bytes, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_dispatch");
  if (rc) return rc;
  // with T == 0 only counts and offsets are written (zeros); the per-assignment arrays may be null
  if (!counts || !offsets || !ws || (shape->T > 0 && (!topk_idx || !row_of || !src_of || !X || !Xp))) {
    set_error("moe_dispatch: null pointer");
    return MOE_EINVAL;
  }
  if (!aligned16(X) || !aligned16(Xp) || !aligned16(ws)) {
    set_error("moe_dispatch: X, Xp and ws must be 16-byte aligned");
    return MOE_EINVAL;
  }
  if (ws_bytes < moe_dispatch_workspace_bytes(shape)) {
    set_error("moe_dispatch: workspace of %zu bytes, need %zu", ws_bytes, moe_dispatch_workspace_bytes(shape));
    return MOE_EWS;
  }
  dispatch_launch(shape, X, topk_idx, counts, offsets, row_of, src_of, Xp, (int32_t*)ws, (hipStream_t)stream);
  return launch_status("moe_dispatch");
}

extern "C" int moe_dispatch_static(const moe_shape_t* shape, const void* X, const int32_t* topk_idx, int32_t* counts,
                                   int32_t* offsets, int32_t* row_of, int32_t* src_of, void* Xp, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_dispatch_static");
  if (rc) return rc;
  if (!counts || !offsets || (shape->T > 0 && (!topk_idx || !row_of || !src_of || !X || !Xp))) {
    set_error("moe_dispatch_static: null pointer");
    return MOE_EINVAL;
  }
  if (!aligned16(X) || !aligned16(Xp)) {
    set_error("moe_dispatch_static: X and Xp must be 16-byte aligned");
    return MOE_EINVAL;
  }
  const size_t need = moe_dispatch_workspace_bytes(shape);
  if (need > kStaticHistInts * sizeof(int32_t)) {
    set_error("moe_dispatch_static: ceil(T*k / 256) * E = %zu counters exceed the built-in scratch of %zu; use "
              "moe_dispatch with a workspace", need / sizeof(int32_t), kStaticHistInts);
    return MOE_EWS;
  }
  int32_t* hist = static_scratch();
  if (!hist) return MOE_ELAUNCH;
  dispatch_launch(shape, X, topk_idx, counts, offsets, row_of, src_of, Xp, hist, (hipStream_t)stream);
  return launch_status("moe_dispatch_static");
}
