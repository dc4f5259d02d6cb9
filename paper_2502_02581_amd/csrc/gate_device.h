// Device code of the gate shared by the route kernels and the fused route + dispatch prologue.
#pragma once

#include "moe_common.h"

namespace moe {

// One token on one wavefront: lane l holds logits l, l + 64, ...; k rounds of wave-wide arg-max.
// Lane j < k ends up with the j-th selected expert and its weight (written to topk_idx/topk_w); the
// logits stay in v for the caller.
template <int R>  // logits per lane, E <= 64*R
__device__ __forceinline__ void route_token(const float* __restrict__ row, int lane, int E, int k, int gate, int renorm,
                                            float (&v)[R], int& sel_e_out, float& w_out) {
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
  sel_e_out = sel_e;
  w_out = p;
}

// ---- auxiliary load-balancing loss: L = alpha E sum_e f_e P_e, f_e = counts[e] / (T k),
// P_e = mean over tokens of expert e's share of the gate's scores (softmax, or sigmoid scores
// divided by their sum over the E experts).  Same mapping as route_kernel: one wavefront per token,
// lane l holds experts l, l + 64, ...
// (from logits already in registers: v[r] = logit of expert lane + 64 r, -inf beyond E)
template <int R>
__device__ __forceinline__ void gate_shares_of(const float (&v)[R], int lane, int E, int gate, float (&s)[R],
                                               float (&p)[R], float& inv_tot) {
  float tot = 0.f;
  if (gate == MOE_GATE_SOFTMAX) {
    float m = v[0];
#pragma unroll
    for (int r = 1; r < R; r++) m = fmaxf(m, v[r]);
    m = wave_max(m);
#pragma unroll
    for (int r = 0; r < R; r++) {
      s[r] = lane + 64 * r < E ? expf(v[r] - m) : 0.f;
      tot += s[r];
    }
  } else {
#pragma unroll
    for (int r = 0; r < R; r++) {
      s[r] = lane + 64 * r < E ? 1.f / (1.f + expf(-v[r])) : 0.f;
      tot += s[r];
    }
  }
  inv_tot = 1.f / wave_sum(tot);
#pragma unroll
  for (int r = 0; r < R; r++) p[r] = s[r] * inv_tot;
}
template <int R>
__device__ __forceinline__ void gate_shares(const float* __restrict__ row, int lane, int E, int gate, float (&s)[R],
                                            float (&p)[R], float& inv_tot) {
  float v[R];
#pragma unroll
  for (int r = 0; r < R; r++) v[r] = lane + 64 * r < E ? row[lane + 64 * r] : -INFINITY;
  gate_shares_of<R>(v, lane, E, gate, s, p, inv_tot);
}

}  // namespace moe

// instantiation by the number of logits a lane holds: CALL(R) with E <= 64 * R
#define MOE_BY_EXPERTS(E, CALL) \
  do {                          \
    if ((E) <= 64) CALL(1);     \
    else if ((E) <= 128) CALL(2); \
    else if ((E) <= 256) CALL(4); \
    else if ((E) <= 512) CALL(8); \
    else CALL(16);              \
  } while (0)

