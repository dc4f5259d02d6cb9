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

}  // namespace moe

extern "C" int moe_route(const moe_shape_t* shape, const float* logits, int32_t* topk_idx, float* topk_w,
                         void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_route");
  if (rc) return rc;
  if (!logits || !topk_idx || !topk_w) {
    set_error("moe_route: null pointer");
    return MOE_EINVAL;
  }
  if (shape->T == 0) return MOE_OK;
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
