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
#include <algorithm>
#include <mutex>

#include "gate_device.h"
#include "moe_common.h"

namespace moe {

constexpr int kChunk = 256;  // most assignments per wavefront in steps 1 and 3
constexpr int kShareFloats = 8192;  // LDS floats of the fused prologue for the per-wave share sums

__global__ __launch_bounds__(64) void dispatch_count(const int32_t* __restrict__ topk_idx, int A, int E, int chunk_len,
                                                     int32_t* __restrict__ hist) {
  __shared__ int32_t cnt[MOE_MAX_EXPERTS];
  const int lane = threadIdx.x;
  const int chunk = blockIdx.x;
  for (int e = lane; e < E; e += 64) cnt[e] = 0;
  __syncthreads();
  const int a0 = chunk * chunk_len, a1 = min(A, a0 + chunk_len);
  for (int s = 0; s < chunk_len; s += 64) {
    int a = a0 + s + lane;
    if (a < a1) {
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
// With `partial` (the fused prologue), the block also finishes the auxiliary load-balancing loss: P_e from
// the per-chunk sums of the gate's shares (added in the same fixed order as the counters), then
// L = alpha E sum_e (counts[e] / (T k)) P_e over ascending e.
__global__ __launch_bounds__(1024) void dispatch_scan(int32_t* __restrict__ hist, int n_chunks, int E,
                                                      int32_t* __restrict__ counts,
                                                      int32_t* __restrict__ offsets,
                                                      const float* __restrict__ partial, float* __restrict__ P,
                                                      float* __restrict__ loss, int T, int k, float alpha) {
  __shared__ int32_t sc[MOE_MAX_EXPERTS];
  __shared__ int32_t part[1024];
  __shared__ float fpart[1024];
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
    if (partial) {
      float fs = 0.f;
#pragma unroll 8
      for (int w = w0; w < w1; w++) fs += partial[(size_t)w * E + e_run];
      fpart[c * E + e_run] = fs;
    }
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
  if (partial) {
    __syncthreads();
    float* term = reinterpret_cast<float*>(sc);  // (the scan is done with it)
    if (e < E) {
      float fs = 0.f;
      for (int q = 0; q < C; q++) fs += fpart[q * E + e];
      const float pe = T > 0 ? fs / (float)T : 0.f;
      P[e] = pe;
      term[e] = T > 0 ? pe * ((float)run / ((float)T * (float)k)) : 0.f;
    }
    __syncthreads();
    if (e == 0) {
      float fs = 0.f;
      for (int q = 0; q < E; q++) fs += term[q];
      *loss = alpha * (float)E * fs;
    }
  }
}

// The gate and the first step of the dispatch in one pass over the logits: a block owns one chunk of
// tokens_per_chunk tokens (tokens_per_chunk * k <= kChunk assignments); its wavefronts take the tokens
// of the chunk in turn (route_token), count the selected experts in LDS (integer atomics on counts
// only) and, for the auxiliary loss, add up the gate's shares of their tokens; the waves' sums are
// added in wave order, so the per-chunk sums do not depend on timing.
template <int R>
__global__ __launch_bounds__(1024) void route_hist_kernel(const float* __restrict__ logits, int32_t* __restrict__ topk_idx,
                                                          float* __restrict__ topk_w, int T, int E, int k, int gate,
                                                          int renorm, int tokens_per_chunk, int32_t* __restrict__ hist,
                                                          float* __restrict__ partial) {
  __shared__ int32_t cnt[MOE_MAX_EXPERTS];
  __shared__ float shares[kShareFloats];  // [wave][64 R]: the launcher keeps waves * 64 R within it
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  const int chunk = blockIdx.x;
  for (int e = threadIdx.x; e < E; e += blockDim.x) cnt[e] = 0;
  __syncthreads();
  const int t0 = chunk * tokens_per_chunk, t1 = min(T, t0 + tokens_per_chunk);
  float acc[R];
#pragma unroll
  for (int r = 0; r < R; r++) acc[r] = 0.f;
  for (int t = t0 + wave; t < t1; t += n_waves) {
    float v[R], w;
    int e;
    route_token<R>(logits + (size_t)t * E, lane, E, k, gate, renorm, v, e, w);
    if (lane < k) {
      topk_idx[(size_t)t * k + lane] = e;
      topk_w[(size_t)t * k + lane] = w;
      atomicAdd(&cnt[e], 1);
    }
    if (partial) {
      float s[R], p[R], inv_tot;
      gate_shares_of<R>(v, lane, E, gate, s, p, inv_tot);
#pragma unroll
      for (int r = 0; r < R; r++) acc[r] += p[r];
    }
  }
  if (partial) {
#pragma unroll
    for (int r = 0; r < R; r++)
      if (lane + 64 * r < E) shares[wave * 64 * R + lane + 64 * r] = acc[r];
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    hist[(size_t)chunk * E + e] = cnt[e];
    if (partial) {
      float fs = 0.f;
      for (int wv = 0; wv < n_waves; wv++) fs += shares[wv * 64 * R + e];
      partial[(size_t)chunk * E + e] = fs;
    }
  }
}

__global__ __launch_bounds__(64) void dispatch_rank(const int32_t* __restrict__ topk_idx, int A, int E, int chunk_len,
                                                    const int32_t* __restrict__ hist,
                                                    const int32_t* __restrict__ offsets,
                                                    int32_t* __restrict__ row_of,
                                                    int32_t* __restrict__ src_of) {
  __shared__ int32_t nxt[MOE_MAX_EXPERTS];
  const int lane = threadIdx.x;
  const int chunk = blockIdx.x;
  for (int e = lane; e < E; e += 64) nxt[e] = offsets[e] + hist[(size_t)chunk * E + e];
  __syncthreads();
  const int a0 = chunk * chunk_len, a1 = min(A, a0 + chunk_len);
  const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  for (int s = 0; s < chunk_len; s += 64) {
    const int a = a0 + s + lane;
    int e = -1;
    if (a < a1) {
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
// rank and row copy of a dispatch whose per-chunk histograms `hist` (chunks of chunk_len assignments)
// have been scanned
static void dispatch_place(const moe_shape_t* shape, const void* X, const int32_t* topk_idx, const int32_t* offsets,
                           int32_t* row_of, int32_t* src_of, void* Xp, const int32_t* hist, int chunk_len, int n_chunks,
                           hipStream_t st) {
  const int A = shape->T * shape->k;
  if (n_chunks <= 0) return;
  {
    ProfScope prof("dispatch_rank", st);
    hipLaunchKernelGGL(dispatch_rank, dim3(n_chunks), dim3(64), 0, st, topk_idx, A, shape->E, chunk_len, hist, offsets,
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

// the four launches of a dispatch; `hist` is scratch of n_chunks * E counters (every one is written
// by dispatch_count before anything reads it)
static void dispatch_launch(const moe_shape_t* shape, const void* X, const int32_t* topk_idx, int32_t* counts,
                            int32_t* offsets, int32_t* row_of, int32_t* src_of, void* Xp, int32_t* hist,
                            hipStream_t st) {
  const int A = shape->T * shape->k;
  const int n_chunks = (A + kChunk - 1) / kChunk;
  if (n_chunks > 0) {
    ProfScope prof("dispatch_count", st);
    hipLaunchKernelGGL(dispatch_count, dim3(n_chunks), dim3(64), 0, st, topk_idx, A, shape->E, kChunk, hist);
  }
  {
    ProfScope prof("dispatch_scan", st);
    hipLaunchKernelGGL(dispatch_scan, dim3(1), dim3(1024), 0, st, hist, n_chunks, shape->E, counts, offsets,
                       (const float*)nullptr, (float*)nullptr, (float*)nullptr, 0, 1, 0.f);
  }
  dispatch_place(shape, X, topk_idx, offsets, row_of, src_of, Xp, hist, kChunk, n_chunks, st);
}

// chunks of the fused prologue: whole tokens, at most kChunk assignments, and fewer than that while the
// batch is too small to give every compute unit a chunk (a chunk is a block of the first kernel)
static int prologue_tokens_per_chunk(const moe_shape_t* s) {
  return std::max(1, std::min(kChunk / s->k, (s->T + 255) / 256));
}
static int prologue_chunks(const moe_shape_t* s) {
  const int tpc = prologue_tokens_per_chunk(s);
  return (s->T + tpc - 1) / tpc;
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

extern "C" size_t moe_route_dispatch_workspace_bytes(const moe_shape_t* shape) {
  using namespace moe;
  if (!shape || shape->E < 1 || shape->T < 0 || shape->k < 1) return 0;
  const size_t per = align_up((size_t)std::max(1, prologue_chunks(shape)) * (size_t)shape->E * 4, 256);
  return 2 * per;  // integer histograms, then the share sums of the auxiliary loss
}

extern "C" int moe_route_dispatch(const moe_shape_t* shape, const float* logits, const void* X, float aux_alpha,
                                  int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets,
                                  int32_t* row_of, int32_t* src_of, void* Xp, float* aux_P, float* aux_loss, void* ws,
                                  size_t ws_bytes, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_route_dispatch");
  if (rc) return rc;
  if (!counts || !offsets || !ws || (aux_P != nullptr) != (aux_loss != nullptr) ||
      (shape->T > 0 && (!logits || !topk_idx || !topk_w || !row_of || !src_of || !X || !Xp))) {
    set_error("moe_route_dispatch: null pointer (aux_P and aux_loss go together)");
    return MOE_EINVAL;
  }
  if (!aligned16(X) || !aligned16(Xp) || !aligned16(ws)) {
    set_error("moe_route_dispatch: X, Xp and ws must be 16-byte aligned");
    return MOE_EINVAL;
  }
  const size_t need = moe_route_dispatch_workspace_bytes(shape);
  if (ws_bytes < need) {
    set_error("moe_route_dispatch: workspace of %zu bytes, need %zu", ws_bytes, need);
    return MOE_EWS;
  }
  hipStream_t st = (hipStream_t)stream;
  const int T = shape->T, E = shape->E, k = shape->k;
  const int tpc = prologue_tokens_per_chunk(shape), n_chunks = prologue_chunks(shape);
  int32_t* hist = (int32_t*)ws;
  float* partial = aux_P ? (float*)((char*)ws + need / 2) : nullptr;
  if (n_chunks > 0) {
    ProfScope prof("route_hist_kernel", st);
    // one wavefront per token of the chunk, as many as the share sums leave room for in LDS
#define MOE_ROUTE_HIST(R)                                                                                              \
  do {                                                                                                                 \
    const int waves = std::max(1, std::min(std::min(16, kShareFloats / (64 * R)), tpc));                               \
    hipLaunchKernelGGL(route_hist_kernel<R>, dim3(n_chunks), dim3(64 * waves), 0, st, logits, topk_idx, topk_w, T, E, k, \
                       shape->gate, shape->renorm, tpc, hist, partial);                                                \
  } while (0)
    MOE_BY_EXPERTS(E, MOE_ROUTE_HIST);
#undef MOE_ROUTE_HIST
  }
  {
    ProfScope prof("dispatch_scan", st);
    hipLaunchKernelGGL(dispatch_scan, dim3(1), dim3(1024), 0, st, hist, n_chunks, E, counts, offsets,
                       (const float*)partial, aux_P, aux_loss, T, k, aux_alpha);
  }
  dispatch_place(shape, X, topk_idx, offsets, row_of, src_of, Xp, hist, tpc * k, n_chunks, st);
  return launch_status("moe_route_dispatch");
}
