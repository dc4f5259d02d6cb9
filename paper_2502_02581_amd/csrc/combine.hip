// moe_combine / moe_combine_bwd: the weighted sum of Eq. 3 and its adjoint.
// One block per token; every lane owns 16-byte pieces of the row, accumulates the k
// gathered rows in fp32 and rounds once.  Pure HBM streaming: (k + 1 [+1]) rows in, 1 row out.
// The gathered rows are read exactly once, so their loads carry the streaming hint (without it the
// k*T rows displace each other and the token rows in the caches: 0.46 -> 0.40 ms per step for the
// two combine launches of the DeepSeek-shaped workload).
#include "moe_common.h"

namespace moe {

// K > 0: k known at compile time (all loops unrolled, the k gathered loads of a piece are in flight
// together); K == 0: any k.
template <typename T, int K>
__global__ __launch_bounds__(512) void combine_kernel(const T* __restrict__ Yp,
                                                      const int32_t* __restrict__ row_of,
                                                      const float* __restrict__ topk_w,
                                                      const T* Yadd, T* Y, int d, int k_rt) {
  constexpr int N = Vec16<T>::N;
  constexpr int KM = K > 0 ? K : 1;
  const int k = K > 0 ? K : k_rt;
  const int t = blockIdx.x;
  const int vec_per_row = d / N;
  if (K > 0) {
    const T* src[KM];
    float w[KM];
#pragma unroll
    for (int j = 0; j < KM; j++) {
      src[j] = Yp + (size_t)row_of[(size_t)t * k + j] * d;
      w[j] = topk_w ? topk_w[(size_t)t * k + j] : 1.f;
    }
    for (int c = threadIdx.x; c < vec_per_row; c += blockDim.x) {
      float v[KM][N], acc[N];
#pragma unroll
      for (int j = 0; j < KM; j++) Vec16<T>::load_nt(src[j] + c * N, v[j]);
      if (Yadd) {
        Vec16<T>::load(Yadd + (size_t)t * d + c * N, acc);
      } else {
#pragma unroll
        for (int i = 0; i < N; i++) acc[i] = 0.f;
      }
#pragma unroll
      for (int j = 0; j < KM; j++)
#pragma unroll
        for (int i = 0; i < N; i++) acc[i] = fmaf(w[j], v[j][i], acc[i]);
      Vec16<T>::store(Y + (size_t)t * d + c * N, acc);
    }
  } else {
    for (int c = threadIdx.x; c < vec_per_row; c += blockDim.x) {
      float acc[N];
      if (Yadd) {
        Vec16<T>::load(Yadd + (size_t)t * d + c * N, acc);
      } else {
#pragma unroll
        for (int i = 0; i < N; i++) acc[i] = 0.f;
      }
      for (int j = 0; j < k; j++) {
        const int r = row_of[(size_t)t * k + j];
        const float w = topk_w ? topk_w[(size_t)t * k + j] : 1.f;
        float v[N];
        Vec16<T>::load(Yp + (size_t)r * d + c * N, v);
#pragma unroll
        for (int i = 0; i < N; i++) acc[i] = fmaf(w, v[i], acc[i]);
      }
      Vec16<T>::store(Y + (size_t)t * d + c * N, acc);
    }
  }
}

// dYp rows and the k dot products of one token.  The partial dots stay in registers over the whole
// row; one wave reduction per slot and one exchange through LDS per token.
template <typename T, int K>
__global__ __launch_bounds__(512) void combine_bwd_kernel(const T* __restrict__ dY, const T* __restrict__ Yp,
                                                          const int32_t* __restrict__ row_of,
                                                          const float* __restrict__ topk_w,
                                                          T* __restrict__ dYp, float* __restrict__ dw, int d,
                                                          int k_rt) {
  constexpr int N = Vec16<T>::N;
  constexpr int KM = K > 0 ? K : 1;
  const int k = K > 0 ? K : k_rt;
  __shared__ float part[8][KM > 1 ? KM : 1];
  const int t = blockIdx.x;
  const int vec_per_row = d / N;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (K > 0) {
    size_t row[KM];
    float w[KM], dot[KM];
#pragma unroll
    for (int j = 0; j < KM; j++) {
      row[j] = (size_t)row_of[(size_t)t * k + j] * d;
      w[j] = topk_w[(size_t)t * k + j];
      dot[j] = 0.f;
    }
    for (int c = threadIdx.x; c < vec_per_row; c += blockDim.x) {
      float g[N], y[KM][N];
      Vec16<T>::load(dY + (size_t)t * d + c * N, g);
#pragma unroll
      for (int j = 0; j < KM; j++) Vec16<T>::load_nt(Yp + row[j] + c * N, y[j]);
#pragma unroll
      for (int j = 0; j < KM; j++) {
        float o[N];
#pragma unroll
        for (int i = 0; i < N; i++) {
          o[i] = w[j] * g[i];
          dot[j] = fmaf(g[i], y[j][i], dot[j]);
        }
        Vec16<T>::store(dYp + row[j] + c * N, o);
      }
    }
#pragma unroll
    for (int j = 0; j < KM; j++) {
      const float s = wave_sum(dot[j]);
      if (lane == 0) part[wave][j] = s;
    }
    __syncthreads();
    if (threadIdx.x < KM) {
      float s = 0.f;  // fixed order over the waves of the block
      for (int wv = 0; wv < (int)(blockDim.x >> 6); wv++) s += part[wv][threadIdx.x];
      dw[(size_t)t * k + threadIdx.x] = s;
    }
  } else {
    for (int j = 0; j < k; j++) {
      const size_t r = (size_t)row_of[(size_t)t * k + j] * d;
      const float w = topk_w[(size_t)t * k + j];
      float dot = 0.f;
      for (int c = threadIdx.x; c < vec_per_row; c += blockDim.x) {
        float g[N], y[N], o[N];
        Vec16<T>::load(dY + (size_t)t * d + c * N, g);
        Vec16<T>::load(Yp + r + c * N, y);
#pragma unroll
        for (int i = 0; i < N; i++) {
          o[i] = w * g[i];
          dot = fmaf(g[i], y[i], dot);
        }
        Vec16<T>::store(dYp + r + c * N, o);
      }
      dot = wave_sum(dot);
      if (lane == 0) part[wave][0] = dot;
      __syncthreads();
      if (threadIdx.x == 0) {
        float s = 0.f;
        for (int wv = 0; wv < (int)(blockDim.x >> 6); wv++) s += part[wv][0];
        dw[(size_t)t * k + j] = s;
      }
      __syncthreads();
    }
  }
}

// Threads per token block: the 16-byte pieces of a row are spread over as few equal trips as fit 512
// threads, so that no lane idles in the last trip (d = 7168 in bf16: 896 pieces = 2 trips of 448).
static unsigned row_block_threads(int d, int elems_per_piece) {
  const int pieces = d / elems_per_piece;
  const int trips = (pieces + 511) / 512;
  const int per_trip = (pieces + trips - 1) / trips;
  const int threads = (per_trip + 63) / 64 * 64;
  return (unsigned)(threads < 64 ? 64 : threads);
}

template <typename T>
static void launch_combine(const moe_shape_t* s, const void* Yp, const int32_t* row_of, const float* topk_w,
                           const void* Yadd, void* Y, hipStream_t st) {
  dim3 grid(s->T), block(row_block_threads(s->d, Vec16<T>::N));
#define MOE_COMBINE(K)                                                                                       \
  hipLaunchKernelGGL((combine_kernel<T, K>), grid, block, 0, st, (const T*)Yp, row_of, topk_w, (const T*)Yadd, \
                     (T*)Y, s->d, s->k)
  switch (s->k) {
    case 1: MOE_COMBINE(1); break;
    case 2: MOE_COMBINE(2); break;
    case 4: MOE_COMBINE(4); break;
    case 8: MOE_COMBINE(8); break;
    default: MOE_COMBINE(0); break;
  }
#undef MOE_COMBINE
}

template <typename T>
static void launch_combine_bwd(const moe_shape_t* s, const void* dY, const void* Yp, const int32_t* row_of,
                               const float* topk_w, void* dYp, float* dw, hipStream_t st) {
  dim3 grid(s->T), block(row_block_threads(s->d, Vec16<T>::N));
#define MOE_COMBINE_BWD(K)                                                                                    \
  hipLaunchKernelGGL((combine_bwd_kernel<T, K>), grid, block, 0, st, (const T*)dY, (const T*)Yp, row_of, topk_w, \
                     (T*)dYp, dw, s->d, s->k)
  switch (s->k) {
    case 1: MOE_COMBINE_BWD(1); break;
    case 2: MOE_COMBINE_BWD(2); break;
    case 4: MOE_COMBINE_BWD(4); break;
    case 8: MOE_COMBINE_BWD(8); break;
    default: MOE_COMBINE_BWD(0); break;
  }
#undef MOE_COMBINE_BWD
}

}  // namespace moe

extern "C" int moe_combine(const moe_shape_t* shape, const void* Yp, const int32_t* row_of, const float* topk_w,
                           const void* Yadd, void* Y, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_combine");
  if (rc) return rc;
  if (shape->T == 0) return MOE_OK;
  if (!Yp || !row_of || !Y) {
    set_error("moe_combine: null pointer");
    return MOE_EINVAL;
  }
  if (!aligned16(Yp) || !aligned16(Y) || !aligned16(Yadd)) {
    set_error("moe_combine: Yp, Yadd and Y must be 16-byte aligned");
    return MOE_EINVAL;
  }
  hipStream_t st = (hipStream_t)stream;
  ProfScope prof("combine_kernel", st);
  if (shape->dtype == MOE_F32) launch_combine<float>(shape, Yp, row_of, topk_w, Yadd, Y, st);
  else launch_combine<bf16_t>(shape, Yp, row_of, topk_w, Yadd, Y, st);
  return launch_status("moe_combine");
}

extern "C" int moe_combine_bwd(const moe_shape_t* shape, const void* dY, const void* Yp, const int32_t* row_of,
                               const float* topk_w, void* dYp, float* dw, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_combine_bwd");
  if (rc) return rc;
  if (shape->T == 0) return MOE_OK;
  if (!dY || !Yp || !row_of || !topk_w || !dYp || !dw) {
    set_error("moe_combine_bwd: null pointer");
    return MOE_EINVAL;
  }
  if (!aligned16(dY) || !aligned16(Yp) || !aligned16(dYp)) {
    set_error("moe_combine_bwd: dY, Yp and dYp must be 16-byte aligned");
    return MOE_EINVAL;
  }
  hipStream_t st = (hipStream_t)stream;
  ProfScope prof("combine_bwd_kernel", st);
  if (shape->dtype == MOE_F32) launch_combine_bwd<float>(shape, dY, Yp, row_of, topk_w, dYp, dw, st);
  else launch_combine_bwd<bf16_t>(shape, dY, Yp, row_of, topk_w, dYp, dw, st);
  return launch_status("moe_combine_bwd");
}
