// moe_route: the gate of Eq. 3 -- scores, top-k selection, renormalised combine weights.
// One wavefront per token; lane l holds logits l, l+64, ...; each of the k rounds is a
// wave-wide arg-max by xor-shuffles, so no LDS and no atomics are needed.
#include "moe_common.h"

namespace moe {

template <int R>  // logits per lane, E <= 64*R
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits,
                                                    int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w, int T, int E, int k,
                                                    int gate, int renorm) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const float* row = logits + (size_t)t * E;
  float v[R];
#pragma unroll
  for (int r = 0; r < R; r++) {
    int e = lane + 64 * r;
    v[r] = e < E ? row[e] : -INFINITY;
  }
  uint32_t taken = 0;
#pragma unroll
  for (int r = 0; r < R; r++)
    if (lane + 64 * r >= E) taken |= 1u << r;

  float sel_v = 0.f;
  int sel_e = 0;
  for (int j = 0; j < k; j++) {
    float bv = -INFINITY;
    int be = 0x7fffffff;
#pragma unroll
    for (int r = 0; r < R; r++) {
      bool free_ = !((taken >> r) & 1u);
      if (free_ && (be == 0x7fffffff || v[r] > bv)) {
        bv = v[r];
        be = lane + 64 * r;
      }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
      float ov = __shfl_xor(bv, m, kWave);
      int oe = __shfl_xor(be, m, kWave);
      bool other = (oe != 0x7fffffff) && (be == 0x7fffffff || ov > bv || (ov == bv && oe < be));
      if (other) {
        bv = ov;
        be = oe;
      }
    }
    if ((be & 63) == lane) taken |= 1u << (be >> 6);
    if (lane == j) {
      sel_v = bv;
      sel_e = be;
    }
  }
  // scores of the selected experts
  float p;
  if (gate == MOE_GATE_SOFTMAX) {
    float m = __shfl(sel_v, 0, kWave);  // the first selected logit is the row maximum
    p = expf(sel_v - m);
    if (!renorm) {
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < R; r++)
        if (lane + 64 * r < E) s += expf(v[r] - m);
      s = wave_sum(s);
      p = p / s;
    }
  } else {
    p = 1.f / (1.f + expf(-sel_v));
  }
  if (renorm) {
    float s = wave_sum(lane < k ? p : 0.f);
    p = p / s;
  }
  if (lane < k) {
    topk_idx[(size_t)t * k + lane] = sel_e;
    topk_w[(size_t)t * k + lane] = p;
  }
}

// Backward of the gate with the selection held fixed: dlogits from the gradient dw of the combine
// weights.  Same mapping as route_kernel (one wavefront per token, lane l holds logits l, l+64, ...).
//   renorm:  w_j = s_j / tot, tot = sum_j s_j   =>  ds_j = (dw_j - sum_i dw_i w_i) / tot
//   softmax: dz_e = s_e (ds_e - sum_j s_j ds_j)  (ds_e = 0 for experts that were not selected)
//   sigmoid: dz_e = ds_e s_e (1 - s_e)
template <int R>
__global__ __launch_bounds__(256) void route_bwd_kernel(const float* __restrict__ logits,
                                                        const int32_t* __restrict__ topk_idx,
                                                        const float* __restrict__ dw, float* __restrict__ dlogits,
                                                        int T, int E, int k, int gate, int renorm) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const float* row = logits + (size_t)t * E;
  float v[R], s[R];
#pragma unroll
  for (int r = 0; r < R; r++) {
    const int e = lane + 64 * r;
    v[r] = e < E ? row[e] : -INFINITY;
  }
  float m = 0.f, inv_z = 1.f;
  if (gate == MOE_GATE_SOFTMAX) {
    m = v[0];
#pragma unroll
    for (int r = 1; r < R; r++) m = fmaxf(m, v[r]);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, kWave));
    float z = 0.f;
#pragma unroll
    for (int r = 0; r < R; r++) {
      s[r] = lane + 64 * r < E ? expf(v[r] - m) : 0.f;
      z += s[r];
    }
    inv_z = 1.f / wave_sum(z);
#pragma unroll
    for (int r = 0; r < R; r++) s[r] *= inv_z;
  } else {
#pragma unroll
    for (int r = 0; r < R; r++) s[r] = lane + 64 * r < E ? 1.f / (1.f + expf(-v[r])) : 0.f;
  }
  // lane j < k: the j-th selected expert, its score and the gradient of its weight
  const int my_e = lane < k ? topk_idx[(size_t)t * k + lane] : -1;
  const float my_dw = lane < k ? dw[(size_t)t * k + lane] : 0.f;
  float my_s = 0.f;
  if (lane < k) {
    const float z = row[my_e];
    my_s = gate == MOE_GATE_SOFTMAX ? expf(z - m) * inv_z : 1.f / (1.f + expf(-z));
  }
  float my_ds = my_dw;
  if (renorm) {
    const float tot = wave_sum(my_s);
    const float c = wave_sum(my_dw * my_s) / tot;
    my_ds = lane < k ? (my_dw - c) / tot : 0.f;
  }
  const float dot = gate == MOE_GATE_SOFTMAX ? wave_sum(my_s * my_ds) : 0.f;
  // scatter the k values to the lanes that own those experts
  float ds[R];
#pragma unroll
  for (int r = 0; r < R; r++) ds[r] = 0.f;
  for (int j = 0; j < k; j++) {
    const int e = __shfl(my_e, j, kWave);
    const float g = __shfl(my_ds, j, kWave);
#pragma unroll
    for (int r = 0; r < R; r++)
      if (lane + 64 * r == e) ds[r] = g;
  }
#pragma unroll
  for (int r = 0; r < R; r++) {
    const int e = lane + 64 * r;
    if (e < E) {
      const float dz = gate == MOE_GATE_SOFTMAX ? s[r] * (ds[r] - dot) : ds[r] * s[r] * (1.f - s[r]);
      dlogits[(size_t)t * E + e] = dz;
    }
  }
}

}  // namespace moe

extern "C" int moe_route_bwd(const moe_shape_t* shape, const float* logits, const int32_t* topk_idx, const float* dw,
                             float* dlogits, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_route_bwd");
  if (rc) return rc;
  if (shape->T == 0) return MOE_OK;  // nothing to do (empty tensors may be null)
  if (!logits || !topk_idx || !dw || !dlogits) {
    set_error("moe_route_bwd: null pointer");
    return MOE_EINVAL;
  }
  hipStream_t st = (hipStream_t)stream;
  dim3 grid((shape->T + 3) / 4), block(256);
  const int E = shape->E;
  ProfScope prof("route_bwd_kernel", st);
#define MOE_ROUTE_BWD(R)                                                                                       \
  hipLaunchKernelGGL(route_bwd_kernel<R>, grid, block, 0, st, logits, topk_idx, dw, dlogits, shape->T, E, shape->k, \
                     shape->gate, shape->renorm)
  if (E <= 64) MOE_ROUTE_BWD(1);
  else if (E <= 128) MOE_ROUTE_BWD(2);
  else if (E <= 256) MOE_ROUTE_BWD(4);
  else if (E <= 512) MOE_ROUTE_BWD(8);
  else MOE_ROUTE_BWD(16);
#undef MOE_ROUTE_BWD
  return launch_status("moe_route_bwd");
}

extern "C" int moe_route(const moe_shape_t* shape, const float* logits, int32_t* topk_idx, float* topk_w,
                         void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_route");
  if (rc) return rc;
  if (shape->T == 0) return MOE_OK;  // nothing to do (empty tensors may be null)
  if (!logits || !topk_idx || !topk_w) {
    set_error("moe_route: null pointer");
    return MOE_EINVAL;
  }
  hipStream_t st = (hipStream_t)stream;
  dim3 grid((shape->T + 3) / 4), block(256);
  const int E = shape->E;
  ProfScope prof("route_kernel", st);
#define MOE_ROUTE(R)                                                                                  \
  hipLaunchKernelGGL(route_kernel<R>, grid, block, 0, st, logits, topk_idx, topk_w, shape->T, E, shape->k, \
                     shape->gate, shape->renorm)
  if (E <= 64) MOE_ROUTE(1);
  else if (E <= 128) MOE_ROUTE(2);
  else if (E <= 256) MOE_ROUTE(4);
  else if (E <= 512) MOE_ROUTE(8);
  else MOE_ROUTE(16);
#undef MOE_ROUTE
  return launch_status("moe_route");
}
