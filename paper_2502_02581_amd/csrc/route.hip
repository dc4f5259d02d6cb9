// moe_route: the gate of Eq. 3 -- scores, top-k selection, renormalised combine weights.
// One wavefront per token; lane l holds logits l, l+64, ...; each of the k rounds is a
// wave-wide arg-max by xor-shuffles, so no LDS and no atomics are needed.
#include "gate_device.h"
#include "moe_common.h"

namespace moe {

template <int R>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits,
                                                    int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w, int T, int E, int k,
                                                    int gate, int renorm) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  float v[R], w;
  int e;
  route_token<R>(logits + (size_t)t * E, lane, E, k, gate, renorm, v, e, w);
  if (lane < k) {
    topk_idx[(size_t)t * k + lane] = e;
    topk_w[(size_t)t * k + lane] = w;
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

// ---- auxiliary load-balancing loss (gate_shares: gate_device.h)
// Wave w sums the shares of tokens w, w + n_waves, ... in that order and writes its E partial sums:
// no atomics, the same result on every run.
template <int R>
__global__ __launch_bounds__(256) void aux_partial_kernel(const float* __restrict__ logits, float* __restrict__ partial,
                                                          int T, int E, int gate, int n_waves) {
  const int lane = threadIdx.x & 63;
  const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= n_waves) return;
  float acc[R];
#pragma unroll
  for (int r = 0; r < R; r++) acc[r] = 0.f;
  for (int t = w; t < T; t += n_waves) {
    float s[R], p[R], inv_tot;
    gate_shares<R>(logits + (size_t)t * E, lane, E, gate, s, p, inv_tot);
#pragma unroll
    for (int r = 0; r < R; r++) acc[r] += p[r];
  }
#pragma unroll
  for (int r = 0; r < R; r++)
    if (lane + 64 * r < E) partial[(size_t)w * E + lane + 64 * r] = acc[r];
}

// One block of 1024 threads: P_e from the partial sums, then the loss.  The waves are cut into C equal
// runs (C = 1024 / E rounded down to a power of two); thread (c, e) adds run c of expert e in ascending
// wave order, the C run sums are added in ascending c, the E terms of the loss in ascending e: a fixed
// order throughout.
__global__ __launch_bounds__(1024) void aux_finish_kernel(const float* __restrict__ partial,
                                                          const int32_t* __restrict__ counts, float* __restrict__ P,
                                                          float* __restrict__ loss, int T, int E, int k, float alpha,
                                                          int n_waves) {
  __shared__ float part[1024];
  __shared__ float term[MOE_MAX_EXPERTS];
  int C = 1;
  while (C * 2 * E <= 1024) C *= 2;
  const int c = threadIdx.x / E, e = threadIdx.x - c * E;
  if (c < C) {
    const int per = (n_waves + C - 1) / C;
    const int w0 = c * per, w1 = min(n_waves, w0 + per);
    float sum = 0.f;
#pragma unroll 8
    for (int w = w0; w < w1; w++) sum += partial[(size_t)w * E + e];
    part[c * E + e] = sum;
  }
  __syncthreads();
  if ((int)threadIdx.x < E) {
    float sum = 0.f;
    for (int q = 0; q < C; q++) sum += part[q * E + e];
    const float pe = T > 0 ? sum / (float)T : 0.f;
    P[e] = pe;
    term[e] = T > 0 ? pe * ((float)counts[e] / ((float)T * (float)k)) : 0.f;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float sum = 0.f;
    for (int q = 0; q < E; q++) sum += term[q];
    *loss = alpha * (float)E * sum;
  }
}

// dlogits (+)= dloss * dL/dlogits with the loads held constant:
//   c_e = dloss alpha E f_e / T;  softmax: dz_e = p_e (c_e - sum_j p_j c_j);
//   sigmoid (p = s / S): dz_e = (c_e - sum_j p_j c_j) / S * s_e (1 - s_e)
template <int R>
__global__ __launch_bounds__(256) void aux_bwd_kernel(const float* __restrict__ logits, const int32_t* __restrict__ counts,
                                                      float* __restrict__ dlogits, int T, int E, int gate,
                                                      float scale, int accumulate) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  float s[R], p[R], inv_tot;
  gate_shares<R>(logits + (size_t)t * E, lane, E, gate, s, p, inv_tot);
  float c[R], dot = 0.f;
#pragma unroll
  for (int r = 0; r < R; r++) {
    c[r] = lane + 64 * r < E ? scale * (float)counts[lane + 64 * r] : 0.f;
    dot += p[r] * c[r];
  }
  dot = wave_sum(dot);
#pragma unroll
  for (int r = 0; r < R; r++) {
    const int e = lane + 64 * r;
    if (e < E) {
      const float dz = gate == MOE_GATE_SOFTMAX ? p[r] * (c[r] - dot) : (c[r] - dot) * inv_tot * s[r] * (1.f - s[r]);
      float* o = dlogits + (size_t)t * E + e;
      *o = accumulate ? *o + dz : dz;
    }
  }
}

// The two backward kernels above in one pass over the logits: dlogits = (gate backward from dw) + dloss *
// (gradient of the auxiliary loss with the loads held constant); every element is written once.
template <int R>
__global__ __launch_bounds__(256) void route_aux_bwd_kernel(const float* __restrict__ logits,
                                                            const int32_t* __restrict__ topk_idx,
                                                            const float* __restrict__ dw, const int32_t* __restrict__ counts,
                                                            float* __restrict__ dlogits, int T, int E, int k, int gate,
                                                            int renorm, float scale) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const float* row = logits + (size_t)t * E;
  float v[R], raw[R], p[R], inv_tot;
#pragma unroll
  for (int r = 0; r < R; r++) v[r] = lane + 64 * r < E ? row[lane + 64 * r] : -INFINITY;
  gate_shares_of<R>(v, lane, E, gate, raw, p, inv_tot);
  // the gate's scores: the softmax itself (= the shares), or the sigmoid values
  float s[R];
#pragma unroll
  for (int r = 0; r < R; r++) s[r] = gate == MOE_GATE_SOFTMAX ? p[r] : raw[r];
  // ---- gate backward (as route_bwd_kernel): lane j < k holds the j-th selected expert
  const int my_e = lane < k ? topk_idx[(size_t)t * k + lane] : -1;
  const float my_dw = lane < k ? dw[(size_t)t * k + lane] : 0.f;
  float my_s = 0.f;
  for (int j = 0; j < k; j++) {  // fetch the score of every selected expert from the lane that owns it
    const int e = __shfl(my_e, j, kWave);
    float sv = 0.f;
#pragma unroll
    for (int r = 0; r < R; r++)
      if (lane + 64 * r == e) sv = s[r];
    sv = __shfl(sv, e & 63, kWave);
    if (lane == j) my_s = sv;
  }
  float my_ds = my_dw;
  if (renorm) {
    const float tot = wave_sum(my_s);
    const float c = wave_sum(my_dw * my_s) / tot;
    my_ds = lane < k ? (my_dw - c) / tot : 0.f;
  }
  const float dot = gate == MOE_GATE_SOFTMAX ? wave_sum(my_s * my_ds) : 0.f;
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
  // ---- auxiliary loss (as aux_bwd_kernel): c_e = scale * counts[e]
  float c[R], adot = 0.f;
#pragma unroll
  for (int r = 0; r < R; r++) {
    c[r] = lane + 64 * r < E ? scale * (float)counts[lane + 64 * r] : 0.f;
    adot += p[r] * c[r];
  }
  adot = wave_sum(adot);
#pragma unroll
  for (int r = 0; r < R; r++) {
    const int e = lane + 64 * r;
    if (e < E) {
      const float dz = gate == MOE_GATE_SOFTMAX ? s[r] * (ds[r] - dot) : ds[r] * s[r] * (1.f - s[r]);
      const float az = gate == MOE_GATE_SOFTMAX ? p[r] * (c[r] - adot) : (c[r] - adot) * inv_tot * raw[r] * (1.f - raw[r]);
      dlogits[(size_t)t * E + e] = dz + az;
    }
  }
}

static int aux_waves(int T) { return T < 256 ? T : 256; }

}  // namespace moe

extern "C" size_t moe_aux_loss_workspace_bytes(const moe_shape_t* shape) {
  if (!shape || shape->T < 0 || shape->E < 1) return 0;
  return (size_t)moe::aux_waves(shape->T) * (size_t)shape->E * sizeof(float) + 256;
}

extern "C" int moe_aux_loss(const moe_shape_t* shape, const float* logits, const int32_t* counts, float alpha, float* P,
                            float* loss, void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_aux_loss");
  if (rc) return rc;
  if (!P || !loss || (shape->T > 0 && (!logits || !counts || !ws))) {
    set_error("moe_aux_loss: null pointer");
    return MOE_EINVAL;
  }
  if (ws_bytes < moe_aux_loss_workspace_bytes(shape)) {
    set_error("moe_aux_loss: workspace of %zu bytes, need %zu", ws_bytes, moe_aux_loss_workspace_bytes(shape));
    return MOE_EWS;
  }
  hipStream_t st = (hipStream_t)stream;
  const int T = shape->T, E = shape->E, n_waves = aux_waves(T);
  float* partial = (float*)ws;
  ProfScope prof("aux_loss", st);
  if (n_waves > 0) {
    dim3 grid((n_waves + 3) / 4), block(256);
#define MOE_AUX_PARTIAL(R) \
  hipLaunchKernelGGL(aux_partial_kernel<R>, grid, block, 0, st, logits, partial, T, E, shape->gate, n_waves)
    MOE_BY_EXPERTS(E, MOE_AUX_PARTIAL);
#undef MOE_AUX_PARTIAL
  }
  hipLaunchKernelGGL(aux_finish_kernel, dim3(1), dim3(1024), 0, st, partial, counts, P, loss, T, E, shape->k, alpha, n_waves);
  return launch_status("moe_aux_loss");
}

extern "C" int moe_aux_loss_bwd(const moe_shape_t* shape, const float* logits, const int32_t* counts, float alpha,
                                float dloss, int32_t accumulate, float* dlogits, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_aux_loss_bwd");
  if (rc) return rc;
  if (shape->T == 0) return MOE_OK;  // nothing to do (empty tensors may be null)
  if (!logits || !counts || !dlogits) {
    set_error("moe_aux_loss_bwd: null pointer");
    return MOE_EINVAL;
  }
  hipStream_t st = (hipStream_t)stream;
  const int T = shape->T, E = shape->E;
  // c_e = scale * counts[e]
  const float scale = dloss * alpha * (float)E / ((float)T * (float)shape->k) / (float)T;
  dim3 grid((T + 3) / 4), block(256);
  ProfScope prof("aux_loss_bwd", st);
#define MOE_AUX_BWD(R) \
  hipLaunchKernelGGL(aux_bwd_kernel<R>, grid, block, 0, st, logits, counts, dlogits, T, E, shape->gate, scale, \
                     (int)accumulate)
  MOE_BY_EXPERTS(E, MOE_AUX_BWD);
#undef MOE_AUX_BWD
  return launch_status("moe_aux_loss_bwd");
}

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

extern "C" int moe_route_aux_bwd(const moe_shape_t* shape, const float* logits, const int32_t* topk_idx, const float* dw,
                                 const int32_t* counts, float alpha, float dloss, float* dlogits, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_route_aux_bwd");
  if (rc) return rc;
  if (shape->T == 0) return MOE_OK;  // nothing to do (empty tensors may be null)
  if (!logits || !topk_idx || !dw || !counts || !dlogits) {
    set_error("moe_route_aux_bwd: null pointer");
    return MOE_EINVAL;
  }
  hipStream_t st = (hipStream_t)stream;
  const int T = shape->T, E = shape->E;
  const float scale = dloss * alpha * (float)E / ((float)T * (float)shape->k) / (float)T;
  dim3 grid((T + 3) / 4), block(256);
  ProfScope prof("route_bwd_kernel", st);
#define MOE_ROUTE_AUX_BWD(R)                                                                                        \
  hipLaunchKernelGGL(route_aux_bwd_kernel<R>, grid, block, 0, st, logits, topk_idx, dw, counts, dlogits, T, E, shape->k, \
                     shape->gate, shape->renorm, scale)
  MOE_BY_EXPERTS(E, MOE_ROUTE_AUX_BWD);
#undef MOE_ROUTE_AUX_BWD
  return launch_status("moe_route_aux_bwd");
}
