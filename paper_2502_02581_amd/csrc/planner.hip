// Host-side planners of the paper: overlap degree and sliding-window load estimate (Section 4.2),
// Algorithm 1 (sparse materialization) and Algorithm 3 (topology-aware token dispatching).
// Plain C++ on host memory: no GPU call anywhere in this file.  A placement is an E x D matrix of
// bytes (1: device d holds expert e); devices d*dpn .. d*dpn + dpn - 1 form node d.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "moe_common.h"

namespace moe {

static int check_topology(const char* who, int E, int D, int dpn) {
  if (E < 1 || D < 1 || dpn < 1 || D % dpn != 0) {
    set_error("%s: need E >= 1, D >= 1 and D a multiple of the devices per node (E=%d D=%d dpn=%d)", who, E, D, dpn);
    return MOE_EINVAL;
  }
  return MOE_OK;
}

}  // namespace moe

extern "C" int moe_plan_overlap_degree(double t_attn, double bw, double psi, int32_t* t_out) {
  using namespace moe;
  if (!t_out || !(t_attn >= 0) || !(bw >= 0) || !(psi > 0)) {
    set_error("moe_plan_overlap_degree: need T_attn >= 0, bw >= 0, Psi > 0 and an output");
    return MOE_EINVAL;
  }
  const double t = std::floor(t_attn * bw / psi);
  *t_out = t > 2147483647.0 ? 2147483647 : (int32_t)t;
  return MOE_OK;
}

extern "C" int moe_plan_predict_load(const double* history, int32_t n_iters, int32_t E, int32_t w, double* F) {
  using namespace moe;
  if (!history || !F || n_iters < 1 || E < 1 || w < 1) {
    set_error("moe_plan_predict_load: need history, output, n_iters >= 1, E >= 1, w >= 1");
    return MOE_EINVAL;
  }
  const int n = std::min(n_iters, w);
  const double* last = history + (size_t)(n_iters - n) * E;
  for (int e = 0; e < E; e++) {
    double s = 0.0;
    for (int i = 0; i < n; i++) s += last[(size_t)i * E + e];  // oldest first
    F[e] = s / (double)n;
  }
  return MOE_OK;
}

extern "C" int moe_plan_materialize(int32_t E, int32_t D, int32_t dpn, const uint8_t* P, const double* F, int32_t t,
                                    int32_t m, uint8_t* P_out) {
  using namespace moe;
  int rc = check_topology("moe_plan_materialize", E, D, dpn);
  if (rc) return rc;
  if (!P || !F || !P_out || t < 0 || m < 0) {
    set_error("moe_plan_materialize: null pointer or negative t, m");
    return MOE_EINVAL;
  }
  for (int e = 0; e < E; e++)
    if (!(F[e] >= 0)) {
      set_error("moe_plan_materialize: load of expert %d is negative or not a number", e);
      return MOE_EINVAL;
    }
  t = std::min(t, E);
  m = std::min(m, t);
  if (P_out != P) std::memcpy(P_out, P, (size_t)E * D);
  for (size_t i = 0; i < (size_t)E * D; i++) P_out[i] = P_out[i] ? 1 : 0;
  // the t most loaded experts, descending load, equal loads by ascending id
  std::vector<int> order(E);
  for (int e = 0; e < E; e++) order[e] = e;
  std::partial_sort(order.begin(), order.begin() + t, order.end(),
                    [&](int a, int b) { return F[a] > F[b] || (F[a] == F[b] && a < b); });
  if (t <= m) {  // the overlap window binds: the top-t experts go to every device
    for (int i = 0; i < t; i++) std::memset(P_out + (size_t)order[i] * D, 1, D);
    return MOE_OK;
  }
  // the memory budget binds: replicas in proportion to load, spread over nodes first
  const int n_nodes = D / dpn;
  const int64_t tot_slots = (int64_t)D * m;
  std::vector<int> free_slots(D, m);
  std::vector<uint8_t> node_has(n_nodes);
  double top_load = 0.0;
  for (int i = 0; i < t; i++) top_load += F[order[i]];
  for (int i = 0; i < t; i++) {
    const int e = order[i];
    uint8_t* row = P_out + (size_t)e * D;
    int holders = 0;
    std::fill(node_has.begin(), node_has.end(), 0);
    for (int d = 0; d < D; d++)
      if (row[d]) {
        holders++;
        node_has[d / dpn] = 1;
      }
    int64_t n = 0;
    if (top_load > 0) n = std::max<int64_t>((int64_t)std::floor((double)tot_slots * F[e] / top_load), 1);
    n = std::min<int64_t>(n, D - holders);
    for (int64_t r = 0; r < n; r++) {
      // the device that lacks e, has a free slot, and comes first by
      // (its node already holds e, most free slots, lowest id)
      int best = -1;
      for (int d = 0; d < D; d++) {
        if (row[d] || free_slots[d] <= 0) continue;
        if (best < 0) {
          best = d;
          continue;
        }
        const int hb = node_has[best / dpn], hd = node_has[d / dpn];
        if (hd < hb || (hd == hb && free_slots[d] > free_slots[best])) best = d;
      }
      if (best < 0) break;
      row[best] = 1;
      free_slots[best]--;
      node_has[best / dpn] = 1;
    }
  }
  return MOE_OK;
}

extern "C" int moe_plan_dispatch(int32_t E, int32_t D, int32_t dpn, const uint8_t* Pm, const int32_t* T, int32_t* R) {
  using namespace moe;
  int rc = check_topology("moe_plan_dispatch", E, D, dpn);
  if (rc) return rc;
  if (!Pm || !T || !R) {
    set_error("moe_plan_dispatch: null pointer");
    return MOE_EINVAL;
  }
  for (size_t i = 0; i < (size_t)E * D; i++)
    if (T[i] < 0) {
      set_error("moe_plan_dispatch: negative token count");
      return MOE_EINVAL;
    }
  std::memset(R, 0, (size_t)E * D * D * sizeof(int32_t));
  std::vector<int> holders;   // devices holding the expert, ascending, grouped by node through first[]
  std::vector<int> first(D / dpn + 1);
  holders.reserve(D);
  for (int e = 0; e < E; e++) {
    const uint8_t* row = Pm + (size_t)e * D;
    holders.clear();
    for (int node = 0; node * dpn < D; node++) {
      first[node] = (int)holders.size();
      for (int d = node * dpn; d < (node + 1) * dpn; d++)
        if (row[d]) holders.push_back(d);
    }
    first[D / dpn] = (int)holders.size();
    if (holders.empty()) {
      set_error("moe_plan_dispatch: expert %d is materialized on no device", e);
      return MOE_EINVAL;
    }
    for (int d = 0; d < D; d++) {
      const int32_t x = T[(size_t)e * D + d];
      int32_t* out = R + ((size_t)e * D + d) * D;
      if (row[d]) {  // local dispatching
        out[d] = x;
        continue;
      }
      // holders in the sender's node if there are any (intra-node dispatching), else all holders
      int lo = first[d / dpn], hi = first[d / dpn + 1];
      if (lo == hi) {
        lo = 0;
        hi = (int)holders.size();
      }
      const int cnt = hi - lo, q = x / cnt, rem = x % cnt;
      for (int i = 0; i < cnt; i++) out[holders[lo + i]] = q + (i < rem ? 1 : 0);
    }
  }
  return MOE_OK;
}
