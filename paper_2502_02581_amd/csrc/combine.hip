// moe_combine / moe_combine_bwd: the weighted sum of Eq. 3 and its adjoint.
// One block per token; every lane owns 16-byte pieces of the row, accumulates the k
// gathered rows in fp32 and rounds once.  Pure HBM streaming: (k + 1 [+1]) rows in, 1 row out.
#include "moe_common.h"

namespace moe {

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ Yp,
                                                      const int32_t* __restrict__ row_of,
                                                      const float* __restrict__ topk_w,
                                                      const T* Yadd, T* Y, int d, int k) {
  constexpr int N = Vec16<T>::N;
  const int t = blockIdx.x;
  const int vec_per_row = d / N;
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

template <typename T>
__global__ __launch_bounds__(256) void combine_bwd_kernel(const T* __restrict__ dY, const T* __restrict__ Yp,
                                                          const int32_t* __restrict__ row_of,
                                                          const float* __restrict__ topk_w,
                                                          T* __restrict__ dYp, float* __restrict__ dw, int d,
                                                          int k) {
  constexpr int N = Vec16<T>::N;
  __shared__ float part[4];
  const int t = blockIdx.x;
  const int vec_per_row = d / N;
  for (int j = 0; j < k; j++) {
    const int r = row_of[(size_t)t * k + j];
    const float w = topk_w[(size_t)t * k + j];
    float dot = 0.f;
    for (int c = threadIdx.x; c < vec_per_row; c += blockDim.x) {
      float g[N], y[N], o[N];
      Vec16<T>::load(dY + (size_t)t * d + c * N, g);
      Vec16<T>::load(Yp + (size_t)r * d + c * N, y);
#pragma unroll
      for (int i = 0; i < N; i++) {
        o[i] = w * g[i];
        dot = fmaf(g[i], y[i], dot);
      }
      Vec16<T>::store(dYp + (size_t)r * d + c * N, o);
    }
    dot = wave_sum(dot);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = dot;
    __syncthreads();
    if (threadIdx.x == 0) dw[(size_t)t * k + j] = (part[0] + part[1]) + (part[2] + part[3]);
    __syncthreads();
  }
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
  if (shape->dtype == MOE_F32)
    hipLaunchKernelGGL(combine_kernel<float>, dim3(shape->T), dim3(256), 0, st, (const float*)Yp, row_of, topk_w,
                       (const float*)Yadd, (float*)Y, shape->d, shape->k);
  else
    hipLaunchKernelGGL(combine_kernel<bf16_t>, dim3(shape->T), dim3(256), 0, st, (const bf16_t*)Yp, row_of,
                       topk_w, (const bf16_t*)Yadd, (bf16_t*)Y, shape->d, shape->k);
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
  if (shape->dtype == MOE_F32)
    hipLaunchKernelGGL(combine_bwd_kernel<float>, dim3(shape->T), dim3(256), 0, st, (const float*)dY,
                       (const float*)Yp, row_of, topk_w, (float*)dYp, dw, shape->d, shape->k);
  else
    hipLaunchKernelGGL(combine_bwd_kernel<bf16_t>, dim3(shape->T), dim3(256), 0, st, (const bf16_t*)dY,
                       (const bf16_t*)Yp, row_of, topk_w, (bf16_t*)dYp, dw, shape->d, shape->k);
  return launch_status("moe_combine_bwd");
}
