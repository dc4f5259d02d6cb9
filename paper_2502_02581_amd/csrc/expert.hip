// moe_expert_fwd / moe_expert_bwd: the expert bodies of Eq. 3 (SwiGLU reading of Eq. 1) as
// grouped GEMMs over variable per-expert row counts, and their backward pass.
//
// Forward   F4: [G | U] = Xin_e [Wg_e | Wu_e],  H = silu(G) * U   (dual GEMM, fused epilogue)
//           F5: Yout_e = H_e Wd_e
// Backward  B2a: dH = dYin_e Wd_e^T, epilogue -> dG, dU           (reads the saved G, U)
//           B2b: dXin_e = dG_e Wg_e^T + dU_e Wu_e^T               (two K segments)
//           B3 : dWd_e = H_e^T dYin_e;  [dWg_e | dWu_e] = Xin_e^T [dG_e | dU_e]
// A device-built plan turns the row offsets into a list of row tiles (largest group first,
// groups without rows contribute nothing) so that no host synchronisation is needed.
#include <atomic>

#include "gemm_cores.h"
#include "gemm_plan.h"

namespace moe {

// ------------------------------------------------------------------------------------ plan
__device__ __forceinline__ void block_scan_inclusive(int32_t* sc, int e) {
  for (int step = 1; step < 1024; step <<= 1) {
    int add = e >= step ? sc[e - step] : 0;
    __syncthreads();
    sc[e] += add;
    __syncthreads();
  }
}

// One block of 1024 threads; thread e owns group e.
__global__ __launch_bounds__(1024) void plan_kernel(const int32_t* __restrict__ offsets, int n_groups,
                                                    int n_rows, int BM, Plan pl, int32_t* active_ids,
                                                    int32_t* n_active) {
  __shared__ int32_t cnt[1024], sc[1024], ord[1024], st_[1024];
  const int e = threadIdx.x;
  int c = 0, st = 0;
  if (e < n_groups) {
    if (offsets) {
      st = offsets[e];
      c = offsets[e + 1] - st;
      if (c < 0) c = 0;
    } else {
      c = n_rows;
    }
  }
  cnt[e] = e < n_groups ? c : -1;
  st_[e] = st;
  sc[e] = (e < n_groups && c > 0) ? 1 : 0;
  __syncthreads();
  // Launch order of the groups: descending row count (ties: ascending id), so that the short tiles
  // of the light groups fill the end of a launch.
  int rank = 0;
  if (e < n_groups) {
    for (int o = 0; o < n_groups; o++) {
      int co = cnt[o];
      rank += (co > c) || (co == c && o < e);
    }
    ord[rank] = e;
  }
  __syncthreads();
  st_[e] = st;
  sc[e] = (e < n_groups && c > 0) ? 1 : 0;
  __syncthreads();
  block_scan_inclusive(sc, e);
  const int total_active = sc[1023];
  if (e < n_groups) {
    const int slot = c > 0 ? sc[e] - 1 : -1;
    if (active_ids) {
      if (slot >= 0) active_ids[slot] = e;
      if (e >= total_active) active_ids[e] = -1;
    }
  }
  if (e < n_groups) pl.ginfo[rank] = make_int4(e, c, st, c > 0 ? sc[e] - 1 : -1);
  if (e == 0 && n_active) *n_active = total_active;
  __syncthreads();
  // Row tiles, groups in descending size.  BM > 0: tiles of BM rows.  BM == 0: mixed heights -- full
  // 256-row tiles, and the remainder r of a group cut so that little MFMA work is spent on padding:
  // r > 192: one 256 tile; (160,192]: 128 + 64; (128,160]: 128 + 32; (96,128]: 128; (64,96]: 64 + 32;
  // (32,64]: 64; (0,32]: 32.
  const int g = e < n_groups ? ord[e] : 0;
  const int cg = e < n_groups ? cnt[g] : 0;
  int nt, h0 = 0, h1 = 0;  // heights of the (up to two) remainder tiles
  if (BM > 0) {
    nt = (cg + BM - 1) / BM;
  } else {
    const int r = cg & 255;
    if (r > 192) h0 = 256;
    else if (r > 160) { h0 = 128; h1 = 64; }
    else if (r > 128) { h0 = 128; h1 = 32; }
    else if (r > 96) h0 = 128;
    else if (r > 64) { h0 = 64; h1 = 32; }
    else if (r > 32) h0 = 64;
    else if (r > 0) h0 = 32;
    nt = (cg >> 8) + (h0 > 0) + (h1 > 0);
  }
  sc[e] = nt;
  __syncthreads();
  block_scan_inclusive(sc, e);
  const int base = sc[e] - nt;
  if (BM > 0) {
    for (int i = 0; i < nt; i++) {
      RowTile t;
      t.group = g;
      t.row0_in = st_[g] + i * BM;
      t.rows = min(BM, cg - i * BM);
      t.row0_out = offsets ? t.row0_in : g * n_rows + i * BM;
      pl.tiles[base + i] = t;
    }
  } else {
    int row = 0;
    for (int i = 0; i < nt; i++) {
      const int full = cg >> 8;
      const int h = i < full ? 256 : (i == full ? h0 : h1);
      const int kind = h == 256 ? 0 : h == 128 ? 1 : h == 64 ? 2 : 3;
      RowTile t;
      t.group = g;
      t.row0_in = st_[g] + row;
      t.rows = min(h, cg - row) | (kind << 16);
      t.row0_out = offsets ? t.row0_in : g * n_rows + row;
      pl.tiles[base + i] = t;
      row += h;
    }
  }
  if (e == 1023) *pl.n_tiles = sc[1023];
}

// ------------------------------------------------------------------------------- epilogues
// W consecutive elements (W = 4 or 8) narrowed from / widened to fp32, one or two 16-byte accesses
template <typename T, int W> struct Pack;
template <int W> struct Pack<float, W> {
  __device__ static __forceinline__ void widen(const uint4&, float (&)[W]) {}  // (bf16 only)
  __device__ static __forceinline__ void store(float* p, const float (&v)[W]) {
#pragma unroll
    for (int i = 0; i < W; i += 4) *reinterpret_cast<float4*>(p + i) = make_float4(v[i], v[i + 1], v[i + 2], v[i + 3]);
  }
  __device__ static __forceinline__ void store_nt(float* p, const float (&v)[W]) { store(p, v); }
  __device__ static __forceinline__ void load(const float* p, float (&v)[W]) {
#pragma unroll
    for (int i = 0; i < W; i += 4) {
      float4 f = *reinterpret_cast<const float4*>(p + i);
      v[i] = f.x; v[i + 1] = f.y; v[i + 2] = f.z; v[i + 3] = f.w;
    }
  }
};
template <int W> struct Pack<bf16_t, W> {
  __device__ static __forceinline__ void store(bf16_t* p, const float (&v)[W]) {
    uint32_t w[W / 2];
#pragma unroll
    for (int i = 0; i < W / 2; i++) w[i] = f32x2_to_bf16x2(v[2 * i], v[2 * i + 1]);
    if (W == 4) *reinterpret_cast<uint2*>(p) = make_uint2(w[0], w[1]);
    else *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[W / 2 - 2], w[W / 2 - 1]);
  }
  // the same with a streaming hint: for outputs that nothing on the chip reads again soon
  __device__ static __forceinline__ void store_nt(bf16_t* p, const float (&v)[W]) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
    uint32_t w[W / 2];
#pragma unroll
    for (int i = 0; i < W / 2; i++) w[i] = f32x2_to_bf16x2(v[2 * i], v[2 * i + 1]);
    if (W == 4) {
      u32x2 t = {w[0], w[1]};
      __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(p));
    } else {
      u32x4 t = {w[0], w[1], w[W / 2 - 2], w[W / 2 - 1]};
      __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
    }
  }
  // the same from a 16-byte piece that is already in registers (W == 8)
  __device__ static __forceinline__ void widen(const uint4& t, float (&v)[W]) {
    if constexpr (W == 8) {  // (cores that hand over four values at a time do their own loads)
      const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
      for (int i = 0; i < 4; i++) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      }
    }
  }
  __device__ static __forceinline__ void load(const bf16_t* p, float (&v)[W]) {
    uint32_t w[W / 2];
    if (W == 4) {
      uint2 t = *reinterpret_cast<const uint2*>(p);
      w[0] = t.x; w[1] = t.y;
    } else {
      uint4 t = *reinterpret_cast<const uint4*>(p);
      w[0] = t.x; w[1] = t.y; w[W / 2 - 2] = t.z; w[W / 2 - 1] = t.w;
    }
#pragma unroll
    for (int i = 0; i < W / 2; i++) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

enum { EPI_STORE = 0, EPI_SWIGLU_FWD = 1, EPI_SWIGLU_BWD = 2, EPI_STORE_F32 = 3, EPI_ADD = 4, EPI_GELU_FWD = 5,
       EPI_GELU_BWD = 6 };

// gelu(z) = z Phi(z) and its derivative Phi(z) + z phi(z) (Phi, phi: standard normal distribution
// function and density); the activation of the two-matrix expert.  `e` receives exp(-z^2 / 2).
// fp32 path: the library's erf and exp.  bf16 path (the result is rounded to bf16 anyway): the
// rational-times-exponential approximation of erf (Abramowitz & Stegun 7.1.26, absolute error below
// 1.5e-7) on the hardware's exp and reciprocal, a quarter of the instructions.
template <typename T> __device__ __forceinline__ float normal_cdf_(float z, float& e);
template <> __device__ __forceinline__ float normal_cdf_<float>(float z, float& e) {
  e = expf(-0.5f * z * z);
  return 0.5f * (1.f + erff(z * 0.70710678118654752f));
}
template <> __device__ __forceinline__ float normal_cdf_<bf16_t>(float z, float& e) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(1.f + 0.3275911f * x);
  e = __expf(-x * x);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float half_erfc = 0.5f * poly * e;  // (1 - erf(x)) / 2
  return z < 0.f ? half_erfc : 1.f - half_erfc;
}
template <typename T> __device__ __forceinline__ float gelu_f(float z) {
  float e;
  return z * normal_cdf_<T>(z, e);
}
template <typename T> __device__ __forceinline__ float gelu_grad_f(float z) {
  float e;
  const float cdf = normal_cdf_<T>(z, e);
  return cdf + z * 0.3989422804014327f * e;
}

// precise for the fp32 path; hardware exp and reciprocal where the result is rounded to bf16 anyway
template <typename T> __device__ __forceinline__ float sigmoidf_(float z);
template <> __device__ __forceinline__ float sigmoidf_<float>(float z) { return 1.f / (1.f + expf(-z)); }
template <> __device__ __forceinline__ float sigmoidf_<bf16_t>(float z) {
  return __builtin_amdgcn_rcpf(1.f + __expf(-z));
}

// An epilogue whose global reads the LDS-DMA core may request ahead of time (see EpiAux): `body` does
// the work, with the pieces `pre` has fetched or, handed a null pointer, with loads of its own.
template <class Body, class Pre, class Aux, int N_AUX>
struct EpiWithAux {
  static constexpr int kAux = N_AUX;
  Body body;
  Pre pre;
  __device__ __forceinline__ Aux prefetch(int m, int n) const { return pre(m, n); }
  template <class V> __device__ __forceinline__ void operator()(int m, int n, const V& v) const {
    body(m, n, v, (const Aux*)nullptr);
  }
  template <class V> __device__ __forceinline__ void operator()(int m, int n, const V& v, const Aux& a) const {
    body(m, n, v, &a);
  }
};

// --------------------------------------------------------------------- row-tiled GEMM kernel
// CoreSet::tile<KIND> is the tile core of a tile kind; kinds differ in height only (same BN, BK), so
// one launch serves full tiles and the short tiles of ragged groups.
template <class Core, int NB, int EPI, bool B_KC>
__device__ __forceinline__ void row_gemm_tile(const RowGemm& p, const RowTile& t, int nt, char* smem) {
  typedef typename Core::T T;
  constexpr int BN = Core::BN, BK = Core::BK;
  const int rows = tile_rows(t);
  const int n0 = nt * BN;
  const int n_valid = min(BN, p.N - n0);
  const int a_row0 = p.a_rows_out ? t.row0_out : t.row0_in;
  const int nk = (p.K + BK - 1) / BK;
  // Where the tiles of this block start in each segment of the sum over K (segments: first all of
  // pair 0, then all of pair 1), and how many bytes of valid data follow the tile origins.
  constexpr int64_t es = sizeof(T);
  const int64_t b_tile = (int64_t)t.group * p.b_group + (B_KC ? (int64_t)n0 * p.ldb : (int64_t)n0);
  // gathered A: the operand pointer stays at the origin of the whole matrix and the row map names the rows
  const RowMap amap = {p.a_index, p.a_index ? p.a_index_div : 1, a_row0, rows};
  const int64_t a_tile = p.a_index ? 0 : (int64_t)a_row0 * p.lda;
  const int64_t a_end = ((int64_t)((p.a_index ? p.a_src_rows : rows) - 1) * p.lda + p.K) * es;
  const int64_t b_end = B_KC ? ((int64_t)(n_valid - 1) * p.ldb + p.K) * es : ((int64_t)(p.K - 1) * p.ldb + (p.N - n0)) * es;
  auto segf = [&](int sg) __attribute__((always_inline)) {
    SegSrc<T, NB> s;
    const int pair = sg >= p.n_segs ? 1 : 0;  // at most two pairs
    const int seg = sg - pair * p.n_segs;
    s.a = (const T*)p.A[pair] + a_tile + seg * p.a_seg;
    const int64_t boff = b_tile + seg * p.b_seg;
    s.b[0] = (const T*)p.B[pair] + boff;
    if (NB == 2) s.b[NB - 1] = (const T*)p.Bdual + boff;
    s.k_len = p.K;
    s.a_bytes = a_end;
    s.b_bytes = b_end;
    return s;
  };
  const int c_row0 = p.c_rows_out ? t.row0_out : t.row0_in;
  // W consecutive columns of one row (W = 4 from the fp32 and general cores, 8 from the DMA core)
  // 16-byte pieces the epilogue reads at its own position, requested ahead of time by the LDS-DMA
  // core (bf16): the saved inputs of the activation's derivative, or the output to accumulate into
  constexpr int kAuxLoads = sizeof(T) != 2 ? 0 : EPI == EPI_SWIGLU_BWD ? 2 : (EPI == EPI_GELU_BWD || EPI == EPI_ADD) ? 1 : 0;
  struct Aux {
    uint4 r[kAuxLoads > 0 ? kAuxLoads : 1];
  };
  auto pre = [&](int m, int n) __attribute__((always_inline)) {
    Aux a;
    // out of range: the first piece of the tile, which exists and is never used
    const bool ok = m < rows && n < n_valid;
    const int64_t off = (int64_t)(c_row0 + (ok ? m : 0)) * p.ldc + n0 + (ok ? n : 0);
    const void* src0 = EPI == EPI_ADD ? (const void*)p.out[0] : p.in[0];
    a.r[0] = *reinterpret_cast<const uint4*>((const T*)src0 + off);
    if (kAuxLoads == 2) a.r[kAuxLoads > 1 ? 1 : 0] = *reinterpret_cast<const uint4*>((const T*)p.in[1] + off);
    return a;
  };
  // (all stores carry the streaming hint: every output here is read again only by a later kernel, after
  // gigabytes of other traffic; 2-3 % on the row GEMMs of the Qwen- and stress-shaped workloads)
  auto body = [&](int m, int n, const auto& v, const Aux* aux) __attribute__((always_inline)) {
    constexpr int W = sizeof(v[0]) / sizeof(float);
    if (m >= rows || n >= n_valid) return;
    const int64_t off = (int64_t)(c_row0 + m) * p.ldc + n0 + n;
    if (EPI == EPI_STORE) {
      Pack<T, W>::store_nt((T*)p.out[0] + off, v[0]);
    } else if (EPI == EPI_STORE_F32) {  // fp32 output whatever the operand type (router logits)
      Pack<float, W>::store((float*)p.out[0] + off, v[0]);
    } else if (EPI == EPI_ADD) {        // accumulate into the output
      float o[W];
      if (aux) Pack<T, W>::widen(aux->r[0], o);
      else Pack<T, W>::load((const T*)p.out[0] + off, o);
#pragma unroll
      for (int q = 0; q < W; q++) o[q] += v[0][q];
      Pack<T, W>::store_nt((T*)p.out[0] + off, o);
    } else if (EPI == EPI_GELU_FWD) {    // two-matrix expert: keep the pre-activation, store f of it
      float h[W];
#pragma unroll
      for (int q = 0; q < W; q++) h[q] = gelu_f<T>(v[0][q]);
      Pack<T, W>::store_nt((T*)p.out[0] + off, v[0]);
      Pack<T, W>::store_nt((T*)p.out[2] + off, h);
    } else if (EPI == EPI_GELU_BWD) {    // dZ = dH f'(Z)
      float z[W], dz[W];
      if (aux) Pack<T, W>::widen(aux->r[0], z);
      else Pack<T, W>::load((const T*)p.in[0] + off, z);
      const float sc = p.c_scale ? p.c_scale[p.a_index[a_row0 + m]] : 1.f;
#pragma unroll
      for (int q = 0; q < W; q++) dz[q] = sc * v[0][q] * gelu_grad_f<T>(z[q]);
      Pack<T, W>::store_nt((T*)p.out[0] + off, dz);
    } else if (EPI == EPI_SWIGLU_FWD) {
      float h[W];
#pragma unroll
      for (int q = 0; q < W; q++) h[q] = v[0][q] * sigmoidf_<T>(v[0][q]) * v[NB - 1][q];
      Pack<T, W>::store_nt((T*)p.out[0] + off, v[0]);
      Pack<T, W>::store_nt((T*)p.out[1] + off, v[NB - 1]);
      Pack<T, W>::store_nt((T*)p.out[2] + off, h);
    } else {
      float g[W], u[W], dg[W], du[W];
      if (aux) {
        Pack<T, W>::widen(aux->r[0], g);
        Pack<T, W>::widen(aux->r[kAuxLoads > 1 ? 1 : 0], u);
      } else {
        Pack<T, W>::load((const T*)p.in[0] + off, g);
        Pack<T, W>::load((const T*)p.in[1] + off, u);
      }
      const float sc = p.c_scale ? p.c_scale[p.a_index[a_row0 + m]] : 1.f;
#pragma unroll
      for (int q = 0; q < W; q++) {
        const float s = sigmoidf_<T>(g[q]);
        const float dh = sc * v[0][q];
        du[q] = dh * g[q] * s;
        dg[q] = dh * u[q] * s * (1.f + g[q] * (1.f - s));
      }
      Pack<T, W>::store_nt((T*)p.out[0] + off, dg);
      Pack<T, W>::store_nt((T*)p.out[1] + off, du);
    }
  };
  if constexpr (kAuxLoads > 0) {
    EpiWithAux<decltype(body), decltype(pre), Aux, kAuxLoads> epi{body, pre};
    Core::run(smem, p.n_pairs * p.n_segs, nk, segf, p.lda, p.ldb, rows, n_valid, epi, amap);
  } else {
    auto epi = [&](int m, int n, const auto& v) __attribute__((always_inline)) { body(m, n, v, (const Aux*)nullptr); };
    Core::run(smem, p.n_pairs * p.n_segs, nk, segf, p.lda, p.ldb, rows, n_valid, epi, amap);
  }
}

template <class CoreSet, int NB, int EPI, bool B_KC>
__global__ __launch_bounds__(CoreSet::template tile<0>::NT) void row_gemm_kernel(RowGemm p) {
  extern __shared__ __align__(16) char smem[];
  typedef typename CoreSet::template tile<0> Core0;
  const int ntn = (p.N + Core0::BN - 1) / Core0::BN;
  int mt, nt;
  if (CoreSet::kKinds == 4) {
    // Blocks go to the XCDs round-robin (block b runs on XCD b % 8) and the 32 CUs of an XCD share
    // one L2, so the 32 blocks an XCD holds at a time should read as few different operand tiles as
    // possible.  Tiles are numbered band by band (a band: kBandRows consecutive row tiles), column
    // by column within a band, and each XCD takes runs of 32 consecutive tiles: 4 row tiles x 8
    // column tiles, 12 operand streams for 32 tiles.
    const int per_band = kBandRows * ntn;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int q = ((j >> 5) * 8 + xcd) * 32 + (j & 31);
    const int band = q / per_band, r = q - band * per_band;
    mt = band * kBandRows + r % kBandRows;
    nt = r / kBandRows;
  } else {
    mt = blockIdx.x / ntn;
    nt = blockIdx.x % ntn;
  }
  RowTile t;
  if (p.tiles) {
    if (mt >= *p.n_tiles) return;
    t = p.tiles[mt];
  } else {
    // direct tiling: tiles of one height (on the LDS-DMA path the caller may pick a shorter kind, so
    // that a GEMM with few column tiles still fills the chip)
    const int kind = CoreSet::kKinds == 4 ? p.direct_kind : 0;
    const int bm = CoreSet::kKinds == 4 ? kind_height(kind) : Core0::BM;
    t.group = 0;
    t.row0_in = mt * bm;
    if (t.row0_in >= p.n_rows) return;
    t.rows = min(bm, p.n_rows - t.row0_in) | (kind << 16);
    t.row0_out = t.row0_in;
  }
  MOE_TRACE_BEGIN();
  if (CoreSet::kKinds == 1) {
    row_gemm_tile<Core0, NB, EPI, B_KC>(p, t, nt, smem);
  } else {
    switch (tile_kind(t)) {  // uniform over the block
      case 0: row_gemm_tile<Core0, NB, EPI, B_KC>(p, t, nt, smem); break;
      case 1: row_gemm_tile<typename CoreSet::template tile<1>, NB, EPI, B_KC>(p, t, nt, smem); break;
      case 2: row_gemm_tile<typename CoreSet::template tile<2>, NB, EPI, B_KC>(p, t, nt, smem); break;
      default: row_gemm_tile<typename CoreSet::template tile<3>, NB, EPI, B_KC>(p, t, nt, smem); break;
    }
  }
  MOE_TRACE_ROW_TILE(EPI | (NB << 4) | ((int)B_KC << 8), nt | (tile_kind(t) << 8) | (tile_rows(t) << 16));
}

// ------------------------------------------------------------------- weight-gradient kernel
template <class Core, int NB>
__global__ __launch_bounds__(Core::NT) void w_gemm_kernel(WGemm p) {
  typedef typename Core::T T;
  extern __shared__ __align__(16) char smem[];
  constexpr int BM = Core::BM, BN = Core::BN, BK = Core::BK;
  const int ntn = (p.N + BN - 1) / BN;
  // a block computes n_reps consecutive column tiles of one row of tiles (n_reps > 1 only where a
  // tile is a single short K step: the block's set-up, its group record and the latency of its
  // first loads are then paid once for several tiles, and the stores of one tile overlap the loads
  // of the next)
  const int reps = p.n_reps > 1 ? p.n_reps : 1;
  const int ntb = (ntn + reps - 1) / reps;
  const int rank = blockIdx.y, mt = blockIdx.x / ntb, nt_first = (blockIdx.x % ntb) * reps;
  // {group, rows, first row, compact slot}; without records every group has n_rows rows and its own slot
  const int4 gi = p.ginfo ? p.ginfo[rank] : make_int4(rank, p.n_rows, 0, rank);
  // the record is the same for the whole block: keep it in scalar registers, and with it every
  // address computation of the K loop
  const int g = __builtin_amdgcn_readfirstlane(gi.x), K = __builtin_amdgcn_readfirstlane(gi.y),
            start = __builtin_amdgcn_readfirstlane(gi.z), slot = __builtin_amdgcn_readfirstlane(gi.w);
  if (K <= 0 || K < p.k_min || K > p.k_max) return;
  // single-product kernels serve the two products of a dual GEMM through blockIdx.z
  const int z = NB == 1 ? blockIdx.z : 0;
  const int a_row0 = start + (p.a_per_group ? g * p.n_rows : 0);
  const int b_row0 = start + (p.b_per_group ? g * p.n_rows : 0);
  const int m0 = mt * BM;
  const int m_valid = min(BM, p.M - m0);
  for (int nt = nt_first; nt < min(nt_first + reps, ntn); nt++) {
  const int n0 = nt * BN;
  const int n_valid = min(BN, p.N - n0);
  if (nt > nt_first) __syncthreads();  // the previous tile's epilogue is done with LDS in every wave
  auto segf = [&](int) __attribute__((always_inline)) {  // one segment: the rows of the group
    SegSrc<T, NB> s;
    s.a = (const T*)p.A + (int64_t)a_row0 * p.lda + m0;
    s.b[0] = (const T*)p.B[z] + (int64_t)b_row0 * p.ldb + n0;
    if (NB == 2) s.b[NB - 1] = (const T*)p.B[1] + (int64_t)b_row0 * p.ldb + n0;
    s.k_len = K;
    const int64_t es = sizeof(T);
    s.a_bytes = ((int64_t)(K - 1) * p.lda + (p.M - m0)) * es;
    s.b_bytes = ((int64_t)(K - 1) * p.ldb + (p.N - n0)) * es;
    return s;
  };
  auto epi = [&](int m, int n, const auto& v) __attribute__((always_inline)) {
    constexpr int W = sizeof(v[0]) / sizeof(float);
    if (m >= m_valid || n >= n_valid) return;
    const int64_t off = (int64_t)slot * p.c_slot + (int64_t)(m0 + m) * p.N + n0 + n;
    Pack<T, W>::store_nt((T*)p.C[z] + off, v[0]);
    if (NB == 2) Pack<T, W>::store_nt((T*)p.C[1] + off, v[NB - 1]);
  };
  MOE_TRACE_BEGIN();
  Core::run(smem, 1, (K + BK - 1) / BK, segf, p.lda, p.ldb, m_valid, n_valid, epi, RowMap{nullptr, 1, 0, 0});
  MOE_TRACE_W_TILE(0x1000 | NB | (BM << 4), g, min(K, 0xffff) << 16);
  }
}

// ------------------------------------------------------------------------------ host side
// Three families of tile cores: fp32 FMA (MOE_F32), the general bf16 MFMA core (any d, d_ff that are
// multiples of 8) and the bf16 core with LDS DMA loads (d and d_ff multiples of 64).
enum { PATH_F32 = 0, PATH_BF16 = 1, PATH_BF16_DMA = 2 };
template <int PATH> struct Cores;
template <> struct Cores<PATH_F32> {
  static constexpr int BM = 64, BN = 64;
  template <int NB, bool A_KC, bool B_KC> using core = F32Core<NB, A_KC, B_KC>;
};
template <> struct Cores<PATH_BF16> {
  static constexpr int BM = 128, BN = 128;
  template <int NB, bool A_KC, bool B_KC> using core = MfmaCore<128, 128, NB, A_KC, B_KC, 2, 2>;
};
template <> struct Cores<PATH_BF16_DMA> {
  static constexpr int BM = 256, BN = 256;
  // one block of 4 wavefronts (one per SIMD, each with a 128 x 128 share: the fewest LDS reads and
  // scalar instructions per MFMA, which is what the K loop is short of) computes 256 x 256 outputs
  // (dual GEMMs: 256 x 128 of each product)
  template <int NB, bool A_KC, bool B_KC> using core = MfmaDmaCore<256, 256 / NB, NB, A_KC, B_KC, 2, 2>;
  // weight gradients of groups with few rows: 128 x 128 outputs per product, one tile slot
  template <int NB> using core_light = MfmaDmaCore<128, 128, NB, false, false, 2, 2, 0>;
};
constexpr int kLightGroupRows = 256;  // groups up to this many rows take the light dW kernel
constexpr int kLightReps = 2;         // column tiles per block of that kernel (1: +5 % time on the DeepSeek shape, 8: +3 %)

// The tile cores a row-tiled GEMM launch may use: one for the fp32 and the general bf16 path, four
// heights (256, 128, 64, 32 rows) for the DMA path so that ragged groups waste little MFMA work.
template <int PATH, int NB, bool B_KC> struct RowCores {
  static constexpr int kKinds = 1;
  template <int KIND> using tile = typename Cores<PATH>::template core<NB, true, B_KC>;
};
template <int NB, bool B_KC> struct RowCores<PATH_BF16_DMA, NB, B_KC> {
  static constexpr int kKinds = 4;
  // tile kinds 0..3 are cut for 256, 128, 64 and 32 rows; the last two share the 64-row core (those
  // tiles are bound by streaming the weights, not by MFMA work).  Pipeline depth by height: the
  // 128-row tile fits 3 slots per operand, the 64-row one 4.
  template <int KIND>
  using tile = MfmaDmaCore<(KIND == 0 ? 256 : KIND == 1 ? 128 : 64), 256 / NB, NB, true, B_KC, 2, 2,
                           (KIND == 0 ? 1 : KIND == 1 ? 2 : 3)>;
};

static int pick_path(const moe_shape_t* s) {
  if (s->dtype == MOE_F32) return PATH_F32;
  return (s->d % 64 == 0 && s->d_ff % 64 == 0) ? PATH_BF16_DMA : PATH_BF16;
}

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// A kernel that wants more than 48 KB of dynamic LDS has to be told so once per device (the
// attribute belongs to the kernel's code object on that device); one instance per kernel.
struct LdsAttr {
  std::atomic<uint64_t> done{0};  // bit i: set on device i
  void ensure(const void* kern, int lds_bytes) {
    if (lds_bytes <= 48 * 1024) return;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return;
    const uint64_t bit = 1ull << (dev & 63);
    if (dev < 64 && (done.load(std::memory_order_relaxed) & bit)) return;
    (void)hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (dev < 64) done.fetch_or(bit, std::memory_order_relaxed);
  }
};

// upper bound of the row tiles the plan kernel may emit (BM == 0: mixed heights, at most two
// remainder tiles per group)
static int max_row_tiles(int n_groups, int n_rows, bool shared, int BM) {
  if (BM == 0) return shared ? n_groups * (n_rows / 256 + 2) : n_rows / 256 + 2 * n_groups;
  return shared ? n_groups * ceil_div(n_rows, BM) : ceil_div(n_rows, BM) + n_groups;
}
template <int PATH> constexpr int plan_bm() { return PATH == PATH_BF16_DMA ? 0 : Cores<PATH>::BM; }

template <class CoreSet, int NB, int EPI, bool B_KC>
static void launch_row(const char* label, const RowGemm& p, int max_tiles, hipStream_t st) {
  typedef typename CoreSet::template tile<0> Core;
  const int ntn = ceil_div(p.N, Core::BN);
  const int n_mt = p.tiles ? max_tiles : ceil_div(p.n_rows, CoreSet::kKinds == 4 ? kind_height(p.direct_kind) : Core::BM);
  if (n_mt == 0 || ntn == 0) return;
  auto kern = row_gemm_kernel<CoreSet, NB, EPI, B_KC>;
  static LdsAttr attr;
  attr.ensure((const void*)kern, Core::LDS_BYTES);
  ProfScope prof(label, st);
  // LDS-DMA path: whole bands of kBandRows row tiles, handed out in runs of 32 tiles to 8 XCDs
  const unsigned n_blocks = CoreSet::kKinds == 4 ? (unsigned)ceil_div(ceil_div(n_mt, kBandRows) * kBandRows * ntn, 256) * 256u
                                                 : (unsigned)(n_mt * ntn);
  hipLaunchKernelGGL(kern, dim3(n_blocks), dim3(Core::NT), Core::LDS_BYTES, st, p);
}

template <class Core, int NB>
static void launch_w(const char* label, const WGemm& p, int n_groups, hipStream_t st, int n_products = 1) {
  const int tiles = ceil_div(p.M, Core::BM) * ceil_div(ceil_div(p.N, Core::BN), p.n_reps > 1 ? p.n_reps : 1);
  if (tiles == 0 || n_groups == 0) return;
  auto kern = w_gemm_kernel<Core, NB>;
  static LdsAttr attr;
  attr.ensure((const void*)kern, Core::LDS_BYTES);
  ProfScope prof(label, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)tiles, (unsigned)n_groups, (unsigned)n_products), dim3(Core::NT), Core::LDS_BYTES, st, p);
}

struct FwdArgs {
  int d, F, n_groups, n_rows;
  const int32_t* offsets;
  const void *Xin, *Wg, *Wu, *Wd;
  void *G, *U, *H, *Yout;
  void* ws;
  // gathered input (moe_expert_fwd_gather): Xin is the token matrix [src_rows, d] and grouped row r reads
  // its row src_of[r] / src_div
  const int32_t* src_of = nullptr;
  int src_div = 1, src_rows = 0;
};

template <int PATH>
static void expert_fwd_impl(const FwdArgs& a, hipStream_t st) {
  const bool shared = a.offsets == nullptr;
  const int max_tiles = max_row_tiles(a.n_groups, a.n_rows, shared, plan_bm<PATH>());
  Plan pl = carve_plan(a.ws, a.n_groups, max_tiles);
  {
    ProfScope prof("plan_kernel", st);
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(1024), 0, st, a.offsets, a.n_groups, a.n_rows, plan_bm<PATH>(), pl,
                       (int32_t*)nullptr, (int32_t*)nullptr);
  }
  // F4: dual GEMM with the SwiGLU epilogue, or (two-matrix expert, Wu == NULL) one GEMM with the GELU epilogue
  RowGemm p = {};
  p.tiles = pl.tiles; p.n_tiles = pl.n_tiles; p.n_rows = a.n_rows;
  p.N = a.F; p.K = a.d; p.n_pairs = 1; p.n_segs = 1;
  p.A[0] = a.Xin; p.lda = a.d; p.a_seg = 0; p.a_rows_out = 0;
  p.a_index = a.src_of; p.a_index_div = a.src_div; p.a_src_rows = a.src_rows;
  p.B[0] = a.Wg; p.Bdual = a.Wu; p.ldb = a.F; p.b_group = (int64_t)a.d * a.F; p.b_seg = 0;
  p.out[0] = a.G; p.out[1] = a.U; p.out[2] = a.H; p.ldc = a.F; p.c_rows_out = 1;
  if (a.Wu) launch_row<RowCores<PATH, 2, false>, 2, EPI_SWIGLU_FWD, false>("gemm_fwd_gate_up", p, max_tiles, st);
  else launch_row<RowCores<PATH, 1, false>, 1, EPI_GELU_FWD, false>("gemm_fwd_gate_up", p, max_tiles, st);
  // F5: Yout = H Wd (shared mode: summed over groups through K segments)
  RowGemm q = {};
  q.n_rows = a.n_rows; q.N = a.d; q.K = a.F; q.n_pairs = 1;
  q.A[0] = a.H; q.lda = a.F; q.a_rows_out = 1;
  q.B[0] = a.Wd; q.ldb = a.d;
  q.out[0] = a.Yout; q.ldc = a.d; q.c_rows_out = 0;
  if (shared) {
    q.tiles = nullptr; q.n_segs = a.n_groups; q.a_seg = (int64_t)a.n_rows * a.F; q.b_seg = (int64_t)a.F * a.d;
    q.b_group = 0;
  } else {
    q.tiles = pl.tiles; q.n_tiles = pl.n_tiles; q.n_segs = 1; q.b_group = (int64_t)a.F * a.d;
  }
  launch_row<RowCores<PATH, 1, false>, 1, EPI_STORE, false>("gemm_fwd_down", q, max_tiles, st);
}

struct BwdArgs {
  int d, F, n_groups, n_rows;
  const int32_t* offsets;
  const void *Xin, *Wg, *Wu, *Wd, *G, *U, *H, *dYin;
  void* dXin;
  int32_t *active_ids, *n_active;
  void *dWg, *dWu, *dWd;
  void* ws;
  size_t plan_sz;
  // gathered upstream gradient (moe_expert_bwd_gather): the product dH reads row src_of[r] / src_div of
  // dY [src_rows, d] and scales row r by row_w[src_of[r]]; the weight gradient of Wd still reads dYin
  const void* dY = nullptr;
  const int32_t* src_of = nullptr;
  const float* row_w = nullptr;
  int src_div = 1, src_rows = 0;
};

template <int PATH>
static void expert_bwd_impl(const BwdArgs& a, hipStream_t st) {
  typedef Cores<PATH> C;
  const bool shared = a.offsets == nullptr;
  const size_t es = PATH == PATH_F32 ? 4 : 2;
  const int max_tiles = max_row_tiles(a.n_groups, a.n_rows, shared, plan_bm<PATH>());
  Plan pl = carve_plan(a.ws, a.n_groups, max_tiles);
  const size_t act_rows = (size_t)(shared ? a.n_groups : 1) * a.n_rows;
  char* dG = (char*)a.ws + a.plan_sz;
  char* dU = dG + align_up(act_rows * a.F * es, 256);
  {
    ProfScope prof("plan_kernel", st);
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(1024), 0, st, a.offsets, a.n_groups, a.n_rows, plan_bm<PATH>(), pl,
                       a.active_ids, a.n_active);
  }
  // B2a: dH = dYin Wd^T, epilogue turns it into dG, dU
  RowGemm p = {};
  p.tiles = pl.tiles; p.n_tiles = pl.n_tiles; p.n_rows = a.n_rows;
  p.N = a.F; p.K = a.d; p.n_pairs = 1; p.n_segs = 1;
  p.A[0] = a.dYin; p.lda = a.d; p.a_rows_out = 0;
  if (a.src_of) {
    p.A[0] = a.dY; p.a_index = a.src_of; p.a_index_div = a.src_div; p.a_src_rows = a.src_rows; p.c_scale = a.row_w;
  }
  p.B[0] = a.Wd; p.ldb = a.d; p.b_group = (int64_t)a.F * a.d;
  p.in[0] = a.G; p.in[1] = a.U; p.out[0] = dG; p.out[1] = dU; p.ldc = a.F; p.c_rows_out = 1;
  const bool gated = a.Wu != nullptr;  // two-matrix expert otherwise: dG is dZ, no dU
  if (gated) launch_row<RowCores<PATH, 1, true>, 1, EPI_SWIGLU_BWD, true>("gemm_bwd_dh", p, max_tiles, st);
  else launch_row<RowCores<PATH, 1, true>, 1, EPI_GELU_BWD, true>("gemm_bwd_dh", p, max_tiles, st);
  // B2b: dXin = dG Wg^T + dU Wu^T
  RowGemm q = {};
  q.n_rows = a.n_rows; q.N = a.d; q.K = a.F; q.n_pairs = gated ? 2 : 1;
  q.A[0] = dG; q.A[1] = dU; q.lda = a.F; q.a_rows_out = 1;
  q.B[0] = a.Wg; q.B[1] = a.Wu; q.ldb = a.F;
  q.out[0] = a.dXin; q.ldc = a.d; q.c_rows_out = 0;
  if (shared) {
    q.tiles = nullptr; q.n_segs = a.n_groups; q.a_seg = (int64_t)a.n_rows * a.F; q.b_seg = (int64_t)a.d * a.F;
    q.b_group = 0;
  } else {
    q.tiles = pl.tiles; q.n_tiles = pl.n_tiles; q.n_segs = 1; q.b_group = (int64_t)a.d * a.F;
  }
  launch_row<RowCores<PATH, 1, true>, 1, EPI_STORE, true>("gemm_bwd_dx", q, max_tiles, st);
  // B3: weight gradients, compacted to active groups, largest group first
  WGemm w = {};
  w.ginfo = pl.ginfo; w.n_rows = a.n_rows;
  w.M = a.F; w.N = a.d;
  w.A = a.H; w.lda = a.F; w.a_per_group = shared;
  w.B[0] = a.dYin; w.ldb = a.d; w.b_per_group = 0;
  w.C[0] = a.dWd; w.c_slot = (int64_t)a.F * a.d;
  WGemm v = {};
  v.ginfo = pl.ginfo; v.n_rows = a.n_rows;
  v.M = a.d; v.N = a.F;
  v.A = a.Xin; v.lda = a.d; v.a_per_group = 0;
  v.B[0] = dG; v.B[1] = dU; v.ldb = a.F; v.b_per_group = shared;
  v.C[0] = a.dWg; v.C[1] = a.dWu; v.c_slot = (int64_t)a.d * a.F;
  w.k_min = v.k_min = 1;
  w.k_max = v.k_max = 0x7fffffff;
  if constexpr (PATH == PATH_BF16_DMA) {
    // groups with few rows are bound by writing their gradient, not by MFMA work: they go to a
    // kernel that keeps several blocks per CU in flight
    if (!shared) {
      const int light_rows = MOE_KNOB("MOE_LIGHT_ROWS", kLightGroupRows);
      w.k_min = v.k_min = light_rows + 1;
      WGemm wl_ = w, vl_ = v;
      wl_.k_min = vl_.k_min = 1;
      wl_.k_max = vl_.k_max = light_rows;
      // column tiles per block: at most kLightReps, and the same for every block of a row of tiles (11
      // column tiles go 6 + 5, not 8 + 3: consecutive blocks run on different XCDs, and unequal blocks
      // would load the XCDs unequally)
      const int reps_max = MOE_KNOB("MOE_LIGHT_REPS", kLightReps);
      auto even_reps = [&](int n_cols) {
        const int ntn = ceil_div(n_cols, C::template core_light<1>::BN);
        return ceil_div(ntn, ceil_div(ntn, reps_max));
      };
      wl_.n_reps = even_reps(wl_.N);
      vl_.n_reps = even_reps(vl_.N);
      launch_w<typename C::template core<1, false, false>, 1>("gemm_bwd_dwd", w, a.n_groups, st);
      if (gated) launch_w<typename C::template core<2, false, false>, 2>("gemm_bwd_dwgu", v, a.n_groups, st);
      else launch_w<typename C::template core<1, false, false>, 1>("gemm_bwd_dwgu", v, a.n_groups, st);
      launch_w<typename C::template core_light<1>, 1>("gemm_bwd_dw_light", wl_, a.n_groups, st);
      launch_w<typename C::template core_light<1>, 1>("gemm_bwd_dw_light", vl_, a.n_groups, st, gated ? 2 : 1);
      return;
    }
  }
  launch_w<typename C::template core<1, false, false>, 1>("gemm_bwd_dwd", w, a.n_groups, st);
  if (gated) launch_w<typename C::template core<2, false, false>, 2>("gemm_bwd_dwgu", v, a.n_groups, st);
  else launch_w<typename C::template core<1, false, false>, 1>("gemm_bwd_dwgu", v, a.n_groups, st);
}

static size_t plan_size_for(int n_groups, int n_rows, bool shared) {
  // sized for the smallest row tile of any path, so the query does not depend on the path taken
  const int bound = max_row_tiles(n_groups, n_rows, shared, 64) + max_row_tiles(n_groups, n_rows, shared, 0);
  return align_up(plan_bytes(n_groups, bound + 1), 256);
}

static int check_expert_args(const moe_shape_t* s, int n_groups, int n_rows, const char* who) {
  int rc = check_shape(s, who);
  if (rc) return rc;
  if (n_groups < 1 || n_groups > MOE_MAX_EXPERTS || n_rows < 0 || (int64_t)n_groups * n_rows >= (int64_t)1 << 31) {
    set_error("%s: bad n_groups=%d n_rows=%d", who, n_groups, n_rows);
    return MOE_EINVAL;
  }
  return MOE_OK;
}

}  // namespace moe

extern "C" size_t moe_expert_fwd_workspace_bytes(const moe_shape_t* shape, int32_t n_groups, int32_t n_rows,
                                                 int32_t shared) {
  using namespace moe;
  if (!shape || n_groups < 1 || n_rows < 0) return 0;
  return plan_size_for(n_groups, n_rows, shared != 0);
}

// plan + dG + dU ([n_rows, d_ff] each; shared mode keeps them per group)
extern "C" size_t moe_expert_bwd_workspace_bytes(const moe_shape_t* shape, int32_t n_groups, int32_t n_rows,
                                                 int32_t shared) {
  using namespace moe;
  if (!shape || n_groups < 1 || n_rows < 0) return 0;
  const size_t rows = (size_t)(shared ? n_groups : 1) * (size_t)n_rows;
  return plan_size_for(n_groups, n_rows, shared != 0) +
         2 * align_up(rows * shape->d_ff * elem_size(shape->dtype), 256);
}

extern "C" int moe_expert_fwd(const moe_shape_t* shape, int32_t n_groups, const int32_t* offsets, int32_t n_rows,
                              const void* Xin, const void* Wg, const void* Wu, const void* Wd, void* G, void* U,
                              void* H, void* Yout, void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  int rc = check_expert_args(shape, n_groups, n_rows, "moe_expert_fwd");
  if (rc) return rc;
  if (!Wg || !Wd || !ws || (n_rows > 0 && (!Xin || !G || (Wu && !U) || !H || !Yout))) {
    set_error("moe_expert_fwd: null pointer");
    return MOE_EINVAL;
  }
  const void* ptrs[] = {Xin, Wg, Wu, Wd, G, U, H, Yout, ws};
  for (const void* p : ptrs)
    if (!aligned16(p)) {
      set_error("moe_expert_fwd: every tensor must be 16-byte aligned");
      return MOE_EINVAL;
    }
  if (ws_bytes < moe_expert_fwd_workspace_bytes(shape, n_groups, n_rows, offsets == nullptr)) {
    set_error("moe_expert_fwd: workspace of %zu bytes, need %zu", ws_bytes,
              moe_expert_fwd_workspace_bytes(shape, n_groups, n_rows, offsets == nullptr));
    return MOE_EWS;
  }
  if (n_rows == 0) return MOE_OK;
  FwdArgs a = {shape->d, shape->d_ff, n_groups, n_rows, offsets, Xin, Wg, Wu, Wd, G, U, H, Yout, ws};
  switch (pick_path(shape)) {
    case PATH_F32: expert_fwd_impl<PATH_F32>(a, (hipStream_t)stream); break;
    case PATH_BF16: expert_fwd_impl<PATH_BF16>(a, (hipStream_t)stream); break;
    default: expert_fwd_impl<PATH_BF16_DMA>(a, (hipStream_t)stream); break;
  }
  return launch_status("moe_expert_fwd");
}

extern "C" int moe_expert_bwd(const moe_shape_t* shape, int32_t n_groups, const int32_t* offsets, int32_t n_rows,
                              const void* Xin, const void* Wg, const void* Wu, const void* Wd, const void* G,
                              const void* U, const void* H, const void* dYin, void* dXin, int32_t* active_ids,
                              int32_t* n_active, void* dWg_c, void* dWu_c, void* dWd_c, void* ws,
                              size_t ws_bytes, void* stream) {
  using namespace moe;
  int rc = check_expert_args(shape, n_groups, n_rows, "moe_expert_bwd");
  if (rc) return rc;
  if (!Wg || !Wd || !ws || !active_ids || !n_active || !dWg_c || (Wu && !dWu_c) || !dWd_c ||
      (n_rows > 0 && (!Xin || !G || (Wu && !U) || !H || !dYin || !dXin))) {
    set_error("moe_expert_bwd: null pointer");
    return MOE_EINVAL;
  }
  const void* ptrs[] = {Xin, Wg, Wu, Wd, G, U, H, dYin, dXin, dWg_c, dWu_c, dWd_c, ws};
  for (const void* p : ptrs)
    if (!aligned16(p)) {
      set_error("moe_expert_bwd: every tensor must be 16-byte aligned");
      return MOE_EINVAL;
    }
  const size_t need = moe_expert_bwd_workspace_bytes(shape, n_groups, n_rows, offsets == nullptr);
  if (ws_bytes < need) {
    set_error("moe_expert_bwd: workspace of %zu bytes, need %zu", ws_bytes, need);
    return MOE_EWS;
  }
  BwdArgs a = {shape->d, shape->d_ff, n_groups, n_rows, offsets, Xin, Wg, Wu, Wd, G, U, H, dYin, dXin,
               active_ids, n_active, dWg_c, dWu_c, dWd_c, ws, plan_size_for(n_groups, n_rows, offsets == nullptr)};
  switch (pick_path(shape)) {
    case PATH_F32: expert_bwd_impl<PATH_F32>(a, (hipStream_t)stream); break;
    case PATH_BF16: expert_bwd_impl<PATH_BF16>(a, (hipStream_t)stream); break;
    default: expert_bwd_impl<PATH_BF16_DMA>(a, (hipStream_t)stream); break;
  }
  return launch_status("moe_expert_bwd");
}

// The same two calls reading token rows in place (grouped mode only): see include/moe_hip.h.
extern "C" int moe_expert_fwd_gather(const moe_shape_t* shape, const int32_t* offsets, const int32_t* src_of,
                                     const void* X, const void* Wg, const void* Wu, const void* Wd, void* G, void* U,
                                     void* H, void* Yout, void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_expert_fwd_gather");
  if (rc) return rc;
  const int n_groups = shape->E, n_rows = shape->T * shape->k;
  if (!offsets || !Wg || !Wd || !ws || (n_rows > 0 && (!src_of || !X || !G || (Wu && !U) || !H || !Yout))) {
    set_error("moe_expert_fwd_gather: null pointer");
    return MOE_EINVAL;
  }
  const void* ptrs[] = {X, Wg, Wu, Wd, G, U, H, Yout, ws};
  for (const void* p : ptrs)
    if (!aligned16(p)) {
      set_error("moe_expert_fwd_gather: every tensor must be 16-byte aligned");
      return MOE_EINVAL;
    }
  if ((int64_t)shape->T * shape->d * (int64_t)elem_size(shape->dtype) >= ((int64_t)1 << 32) - 4096) {
    set_error("moe_expert_fwd_gather: X must be smaller than 4 GiB (32-bit byte offsets); use moe_expert_fwd on a permuted copy");
    return MOE_EINVAL;
  }
  const size_t need = moe_expert_fwd_workspace_bytes(shape, n_groups, n_rows, 0);
  if (ws_bytes < need) {
    set_error("moe_expert_fwd_gather: workspace of %zu bytes, need %zu", ws_bytes, need);
    return MOE_EWS;
  }
  if (n_rows == 0) return MOE_OK;
  FwdArgs a = {shape->d, shape->d_ff, n_groups, n_rows, offsets, X, Wg, Wu, Wd, G, U, H, Yout, ws};
  a.src_of = src_of; a.src_div = shape->k; a.src_rows = shape->T;
  switch (pick_path(shape)) {
    case PATH_F32: expert_fwd_impl<PATH_F32>(a, (hipStream_t)stream); break;
    case PATH_BF16: expert_fwd_impl<PATH_BF16>(a, (hipStream_t)stream); break;
    default: expert_fwd_impl<PATH_BF16_DMA>(a, (hipStream_t)stream); break;
  }
  return launch_status("moe_expert_fwd_gather");
}

extern "C" int moe_expert_bwd_gather(const moe_shape_t* shape, const int32_t* offsets, const int32_t* src_of,
                                     const void* Xp, const void* Wg, const void* Wu, const void* Wd, const void* G,
                                     const void* U, const void* H, const void* dY, const float* topk_w, const void* dYp,
                                     void* dXp, int32_t* active_ids, int32_t* n_active, void* dWg_c, void* dWu_c,
                                     void* dWd_c, void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_expert_bwd_gather");
  if (rc) return rc;
  const int n_groups = shape->E, n_rows = shape->T * shape->k;
  if (!offsets || !Wg || !Wd || !ws || !active_ids || !n_active || !dWg_c || (Wu && !dWu_c) || !dWd_c ||
      (n_rows > 0 && (!src_of || !Xp || !G || (Wu && !U) || !H || !dY || !topk_w || !dYp || !dXp))) {
    set_error("moe_expert_bwd_gather: null pointer");
    return MOE_EINVAL;
  }
  const void* ptrs[] = {Xp, Wg, Wu, Wd, G, U, H, dY, dYp, dXp, dWg_c, dWu_c, dWd_c, ws};
  for (const void* p : ptrs)
    if (!aligned16(p)) {
      set_error("moe_expert_bwd_gather: every tensor must be 16-byte aligned");
      return MOE_EINVAL;
    }
  if ((int64_t)shape->T * shape->d * (int64_t)elem_size(shape->dtype) >= ((int64_t)1 << 32) - 4096) {
    set_error("moe_expert_bwd_gather: dY must be smaller than 4 GiB (32-bit byte offsets); use moe_expert_bwd");
    return MOE_EINVAL;
  }
  const size_t need = moe_expert_bwd_workspace_bytes(shape, n_groups, n_rows, 0);
  if (ws_bytes < need) {
    set_error("moe_expert_bwd_gather: workspace of %zu bytes, need %zu", ws_bytes, need);
    return MOE_EWS;
  }
  BwdArgs a = {shape->d, shape->d_ff, n_groups, n_rows, offsets, Xp, Wg, Wu, Wd, G, U, H, dYp, dXp,
               active_ids, n_active, dWg_c, dWu_c, dWd_c, ws, plan_size_for(n_groups, n_rows, false)};
  a.dY = dY; a.src_of = src_of; a.row_w = topk_w; a.src_div = shape->k; a.src_rows = shape->T;
  switch (pick_path(shape)) {
    case PATH_F32: expert_bwd_impl<PATH_F32>(a, (hipStream_t)stream); break;
    case PATH_BF16: expert_bwd_impl<PATH_BF16>(a, (hipStream_t)stream); break;
    default: expert_bwd_impl<PATH_BF16_DMA>(a, (hipStream_t)stream); break;
  }
  return launch_status("moe_expert_bwd_gather");
}

// ------------------------------------------------------------------------------------ router
// The gating network read as one linear map: logits = X Wr, and its adjoint.  E is arbitrary, so
// the GEMMs run on copies padded to Ep = E rounded up to 64 columns (zeros), which live in the
// workspace; when E is already a multiple of 64 the caller's buffers are used directly.
namespace moe {

template <typename TI, typename TO>
__device__ __forceinline__ TO cvt_elem(TI v);
template <> __device__ __forceinline__ float cvt_elem<float, float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t cvt_elem<bf16_t, bf16_t>(bf16_t v) { return v; }
template <> __device__ __forceinline__ bf16_t cvt_elem<float, bf16_t>(float v) { return f32_to_bf16(v); }

// dst[r][c] = c < cols_in ? src[r][c] : 0 for c < cols_out (cols_out >= cols_in: pad; the other way: strip)
template <typename TI, typename TO>
__global__ __launch_bounds__(256) void recolumn_kernel(const TI* __restrict__ src, TO* __restrict__ dst, int64_t rows,
                                                       int cols_in, int cols_out) {
  const int64_t n = rows * cols_out;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / cols_out;
    const int c = (int)(i - r * cols_out);
    dst[i] = c < cols_in ? cvt_elem<TI, TO>(src[r * cols_in + c]) : cvt_elem<TI, TO>(TI(0));
  }
}
template <typename TI, typename TO>
static void recolumn(const char* label, const void* src, void* dst, int64_t rows, int cols_in, int cols_out, hipStream_t st) {
  const int64_t n = rows * cols_out;
  if (n == 0) return;
  ProfScope prof(label, st);
  hipLaunchKernelGGL((recolumn_kernel<TI, TO>), dim3((unsigned)std::min<int64_t>((n + 255) / 256, 4096)), dim3(256), 0, st,
                     (const TI*)src, (TO*)dst, rows, cols_in, cols_out);
}

static int router_path(const moe_shape_t* s) {
  if (s->dtype == MOE_F32) return PATH_F32;
  return s->d % 64 == 0 ? PATH_BF16_DMA : PATH_BF16;
}
static int padded_experts(const moe_shape_t* s) { return (s->E + 63) / 64 * 64; }

template <int PATH>
static void router_fwd_impl(const moe_shape_t* s, const void* X, const void* Wr, float* logits, char* ws, hipStream_t st) {
  typedef typename Cores<PATH>::template core<1, true, false>::T T;
  const int Ep = padded_experts(s);
  const bool padded = Ep != s->E;
  const void* B = Wr;
  float* out = logits;
  if (padded) {
    T* WrP = (T*)ws;
    out = (float*)(ws + align_up((size_t)s->d * Ep * sizeof(T), 256));
    recolumn<T, T>("router_pad", Wr, WrP, s->d, s->E, Ep, st);
    B = WrP;
  }
  RowGemm p = {};
  p.n_rows = s->T; p.direct_kind = 2;  // 64-row tiles: E is small, so the rows have to fill the chip
  p.N = Ep; p.K = s->d; p.n_pairs = 1; p.n_segs = 1;
  p.A[0] = X; p.lda = s->d;
  p.B[0] = B; p.ldb = Ep;
  p.out[0] = out; p.ldc = Ep;
  launch_row<RowCores<PATH, 1, false>, 1, EPI_STORE_F32, false>("gemm_router_fwd", p, 0, st);
  if (padded) recolumn<float, float>("router_pad", out, logits, s->T, Ep, s->E, st);
}

template <int PATH>
static void router_bwd_impl(const moe_shape_t* s, const void* X, const void* Wr, const float* dlogits, void* dWr, void* dX,
                            bool accumulate, char* ws, hipStream_t st) {
  typedef typename Cores<PATH>::template core<1, true, false>::T T;
  typedef Cores<PATH> C;
  const int Ep = padded_experts(s);
  const bool padded = Ep != s->E;
  // workspace: dlogits in the operand type [T, Ep]; then, when padded, Wr [d, Ep] and dWr [d, Ep]
  T* dlP = (T*)ws;
  char* q0 = ws + align_up((size_t)s->T * Ep * sizeof(T), 256);
  T* WrP = (T*)q0;
  T* dWrP = (T*)(q0 + align_up((size_t)s->d * Ep * sizeof(T), 256));
  recolumn<float, T>("router_pad", dlogits, dlP, s->T, s->E, Ep, st);
  const void* B = Wr;
  void* dW = dWr;
  if (padded) {
    recolumn<T, T>("router_pad", Wr, WrP, s->d, s->E, Ep, st);
    B = WrP;
    dW = dWrP;
  }
  // dWr = X^T dlogits  (one group of T rows)
  WGemm w = {};
  w.ginfo = nullptr; w.n_rows = s->T;
  w.M = s->d; w.N = Ep;
  w.A = X; w.lda = s->d; w.a_per_group = 0;
  w.B[0] = dlP; w.ldb = Ep; w.b_per_group = 0;
  w.C[0] = dW; w.c_slot = (int64_t)s->d * Ep;
  w.k_min = 1; w.k_max = 0x7fffffff;
  launch_w<typename C::template core<1, false, false>, 1>("gemm_router_dw", w, 1, st);
  if (padded) recolumn<T, T>("router_pad", dWrP, dWr, s->d, Ep, s->E, st);
  // dX (+)= dlogits Wr^T
  RowGemm p = {};
  p.n_rows = s->T; p.direct_kind = 0;
  p.N = s->d; p.K = Ep; p.n_pairs = 1; p.n_segs = 1;
  p.A[0] = dlP; p.lda = Ep;
  p.B[0] = B; p.ldb = Ep;
  p.out[0] = dX; p.ldc = s->d;
  if (accumulate) launch_row<RowCores<PATH, 1, true>, 1, EPI_ADD, true>("gemm_router_dx", p, 0, st);
  else launch_row<RowCores<PATH, 1, true>, 1, EPI_STORE, true>("gemm_router_dx", p, 0, st);
}

}  // namespace moe

extern "C" size_t moe_router_fwd_workspace_bytes(const moe_shape_t* shape) {
  using namespace moe;
  if (!shape || shape->E < 1 || shape->d < 1 || shape->T < 0) return 0;
  const int Ep = padded_experts(shape);
  if (Ep == shape->E) return 256;
  return align_up((size_t)shape->d * Ep * elem_size(shape->dtype), 256) + align_up((size_t)shape->T * Ep * 4, 256);
}

extern "C" size_t moe_router_bwd_workspace_bytes(const moe_shape_t* shape) {
  using namespace moe;
  if (!shape || shape->E < 1 || shape->d < 1 || shape->T < 0) return 0;
  const int Ep = padded_experts(shape);
  const size_t es = elem_size(shape->dtype);
  return align_up((size_t)shape->T * Ep * es, 256) + 2 * align_up((size_t)shape->d * Ep * es, 256);
}

extern "C" int moe_router_fwd(const moe_shape_t* shape, const void* X, const void* Wr, float* logits, void* ws,
                              size_t ws_bytes, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_router_fwd");
  if (rc) return rc;
  if (shape->T == 0) return MOE_OK;
  if (!X || !Wr || !logits || !ws) {
    set_error("moe_router_fwd: null pointer");
    return MOE_EINVAL;
  }
  if (!aligned16(X) || !aligned16(Wr) || !aligned16(logits) || !aligned16(ws)) {
    set_error("moe_router_fwd: every tensor must be 16-byte aligned");
    return MOE_EINVAL;
  }
  if (ws_bytes < moe_router_fwd_workspace_bytes(shape)) {
    set_error("moe_router_fwd: workspace of %zu bytes, need %zu", ws_bytes, moe_router_fwd_workspace_bytes(shape));
    return MOE_EWS;
  }
  switch (router_path(shape)) {
    case PATH_F32: router_fwd_impl<PATH_F32>(shape, X, Wr, logits, (char*)ws, (hipStream_t)stream); break;
    case PATH_BF16: router_fwd_impl<PATH_BF16>(shape, X, Wr, logits, (char*)ws, (hipStream_t)stream); break;
    default: router_fwd_impl<PATH_BF16_DMA>(shape, X, Wr, logits, (char*)ws, (hipStream_t)stream); break;
  }
  return launch_status("moe_router_fwd");
}

extern "C" int moe_router_bwd(const moe_shape_t* shape, const void* X, const void* Wr, const float* dlogits, void* dWr,
                              void* dX, int32_t accumulate, void* ws, size_t ws_bytes, void* stream) {
  using namespace moe;
  int rc = check_shape(shape, "moe_router_bwd");
  if (rc) return rc;
  if (!Wr || !dWr || !ws || (shape->T > 0 && (!X || !dlogits || !dX))) {
    set_error("moe_router_bwd: null pointer");
    return MOE_EINVAL;
  }
  if (!aligned16(X) || !aligned16(Wr) || !aligned16(dlogits) || !aligned16(dWr) || !aligned16(dX) || !aligned16(ws)) {
    set_error("moe_router_bwd: every tensor must be 16-byte aligned");
    return MOE_EINVAL;
  }
  if (ws_bytes < moe_router_bwd_workspace_bytes(shape)) {
    set_error("moe_router_bwd: workspace of %zu bytes, need %zu", ws_bytes, moe_router_bwd_workspace_bytes(shape));
    return MOE_EWS;
  }
  if (shape->T == 0) {  // no tokens: the weight gradient is zero, there is no dX
    if (shape->dtype == MOE_F32) recolumn<float, float>("router_pad", nullptr, dWr, shape->d, 0, shape->E, (hipStream_t)stream);
    else recolumn<bf16_t, bf16_t>("router_pad", nullptr, dWr, shape->d, 0, shape->E, (hipStream_t)stream);
    return launch_status("moe_router_bwd");
  }
  switch (router_path(shape)) {
    case PATH_F32: router_bwd_impl<PATH_F32>(shape, X, Wr, dlogits, dWr, dX, accumulate != 0, (char*)ws, (hipStream_t)stream); break;
    case PATH_BF16: router_bwd_impl<PATH_BF16>(shape, X, Wr, dlogits, dWr, dX, accumulate != 0, (char*)ws, (hipStream_t)stream); break;
    default: router_bwd_impl<PATH_BF16_DMA>(shape, X, Wr, dlogits, dWr, dX, accumulate != 0, (char*)ws, (hipStream_t)stream); break;
  }
  return launch_status("moe_router_bwd");
}

MOE_TRACE_DEFINE_READER
