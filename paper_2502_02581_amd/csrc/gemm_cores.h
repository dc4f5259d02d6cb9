// Tile cores of the grouped GEMMs: an fp32 FMA core (correctness path for MOE_F32) and a
// bf16 MFMA core for gfx950 (v_mfma_f32_32x32x16_bf16, operands staged through LDS).
//
// Both cores compute, for one block, acc[nb][..] = sum over iterations of A_tile * B_tile(nb)
// and hand groups of four consecutive columns to an epilogue functor:
//     epi(m, n, vals)   m, n relative to the block tile;  vals[nb][0..3] = C[m][n..n+3]
// A source iterator supplies, per K iteration, the base pointers and the valid extents.
#pragma once

#include "moe_common.h"

namespace moe {

// What one K iteration reads.  Pointers are already offset to the tile's first row/column;
// "kc" (K-contiguous) operands are [rows][K] row-major, otherwise [K][rows] row-major.
template <typename T, int NB>
struct IterSrc {
  const T* a;        // A tile origin for this iteration (k offset included)
  const T* b[NB];    // B tile origin(s)
  int k_left;        // valid K elements from this origin on
};

// ------------------------------------------------------------------------------ fp32 core
template <int NB, bool A_KC, bool B_KC>
struct F32Core {
  typedef float T;
  static constexpr int BM = 64, BN = 64, BK = 16, NT = 256;
  static constexpr int LD = 64 + 4;
  static constexpr int LDS_BYTES = (BK * LD + NB * BK * LD) * 4;

  template <class SrcFn, class Epi>
  __device__ static void run(char* smem, int n_iters, SrcFn src, int64_t lda, int64_t ldb, int m_valid,
                             int n_valid, Epi epi) {
    float* As = (float*)smem;            // [BK][LD]  (k major)
    float* Bs = As + BK * LD;            // [NB][BK][LD]
    const int tid = threadIdx.x;
    const int ty = tid / 16, tx = tid % 16;
    float acc[NB][4][4];
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[nb][i][j] = 0.f;

    for (int it = 0; it < n_iters; it++) {
      IterSrc<float, NB> s = src(it);
      for (int idx = tid; idx < BM * BK; idx += NT) {
        int m, k;
        if (A_KC) { m = idx / BK; k = idx % BK; } else { k = idx / BM; m = idx % BM; }
        float v = 0.f;
        if (m < m_valid && k < s.k_left) v = A_KC ? s.a[(int64_t)m * lda + k] : s.a[(int64_t)k * lda + m];
        As[k * LD + m] = v;
      }
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
        for (int idx = tid; idx < BN * BK; idx += NT) {
          int n, k;
          if (B_KC) { n = idx / BK; k = idx % BK; } else { k = idx / BN; n = idx % BN; }
          float v = 0.f;
          if (n < n_valid && k < s.k_left) v = B_KC ? s.b[nb][(int64_t)n * ldb + k] : s.b[nb][(int64_t)k * ldb + n];
          Bs[(nb * BK + k) * LD + n] = v;
        }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < BK; k++) {
        float a[4], b[NB][4];
#pragma unroll
        for (int i = 0; i < 4; i++) a[i] = As[k * LD + ty * 4 + i];
#pragma unroll
        for (int nb = 0; nb < NB; nb++)
#pragma unroll
          for (int j = 0; j < 4; j++) b[nb][j] = Bs[(nb * BK + k) * LD + tx * 4 + j];
#pragma unroll
        for (int nb = 0; nb < NB; nb++)
#pragma unroll
          for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) acc[nb][i][j] = fmaf(a[i], b[nb][j], acc[nb][i][j]);
      }
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
      float vals[NB][4];
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
#pragma unroll
        for (int j = 0; j < 4; j++) vals[nb][j] = acc[nb][i][j];
      epi(ty * 4 + i, tx * 4, vals);
    }
  }
};

// ------------------------------------------------------------------------------ bf16 MFMA core
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(8))) short short8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// LDS layouts (bf16 elements), BK = 64:
//  K-contiguous operand: [rows][64], the eight 16-byte pieces of a row are XOR-swizzled with
//    (row/2)%8 so that the 16 rows one ds_read_b128 phase touches fall into distinct banks.
//  row-contiguous operand ([K][rows] in memory): [64][rows + 32]; the 64-byte pad moves the four
//    k rows of a transposing read (ds_read_b64_tr_b16) to four different bank quarters.
template <int BM_, int BN_, int NB, bool A_KC, bool B_KC>
struct MfmaCore {
  typedef bf16_t T;
  static constexpr int BM = BM_, BN = BN_, BK = 64, NT = 256;
  static constexpr int WM = 2, WN = 2;
  static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  static constexpr int PAD = 32;
  static constexpr int A_LD = A_KC ? BK : BM + PAD;
  static constexpr int B_LD = B_KC ? BK : BN + PAD;
  static constexpr int A_ELEMS = A_KC ? BM * BK : BK * A_LD;
  static constexpr int B_ELEMS = B_KC ? BN * BK : BK * B_LD;
  static constexpr int LDS_BYTES = (A_ELEMS + NB * B_ELEMS) * 2;
  static constexpr int A_VEC = BM * BK / 8 / NT;
  static constexpr int B_VEC = BN * BK / 8 / NT;
  static_assert(BM % 64 == 0 && BN % 64 == 0, "tile must be a multiple of 64");

  // ---- global -> registers (16 bytes per access), zero outside the valid extents
  template <int ROWS, int NVEC, bool KC>
  __device__ static __forceinline__ void gload(const bf16_t* base, int64_t ld, int rows_valid, int k_left,
                                               uint4 (&r)[NVEC]) {
#pragma unroll
    for (int i = 0; i < NVEC; i++) {
      const int v = threadIdx.x + i * NT;
      int row, kk;
      if (KC) { row = v / (BK / 8); kk = (v % (BK / 8)) * 8; }
      else { kk = v / (ROWS / 8); row = (v % (ROWS / 8)) * 8; }
      const bool ok = row < rows_valid && kk < k_left;
      const bf16_t* p = KC ? base + (int64_t)row * ld + kk : base + (int64_t)kk * ld + row;
      r[i] = ok ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
    }
  }
  // ---- registers -> LDS
  template <int ROWS, int NVEC, bool KC>
  __device__ static __forceinline__ void sstore(bf16_t* lds, const uint4 (&r)[NVEC]) {
#pragma unroll
    for (int i = 0; i < NVEC; i++) {
      const int v = threadIdx.x + i * NT;
      int off;
      if (KC) {
        const int row = v / (BK / 8), c = v % (BK / 8);
        off = row * BK + ((c ^ ((row >> 1) & 7)) << 3);
      } else {
        const int kk = v / (ROWS / 8), c = v % (ROWS / 8);
        off = kk * (ROWS + PAD) + c * 8;
      }
      *reinterpret_cast<uint4*>(lds + off) = r[i];
    }
  }
  // ---- LDS -> MFMA fragment: lane l holds k = 16*ks + 8*(l/32) + 0..7 of row (row0 + l%32)
  template <int ROWS, bool KC>
  __device__ static __forceinline__ bf16x8_t frag(const bf16_t* lds, int row0, int ks) {
    const int lane = threadIdx.x & 63;
    if (KC) {
      const int row = row0 + (lane & 31);
      const int c = ks * 2 + (lane >> 5);
      const uint4 v = *reinterpret_cast<const uint4*>(lds + row * BK + ((c ^ ((row >> 1) & 7)) << 3));
      return __builtin_bit_cast(bf16x8_t, v);
    } else {
      // transposing read: within 16 lanes, lane s reads 4 consecutive rows-elements at
      // k = kb + s/4, column 4*(s%4); it receives k = kb..kb+3 of column s.
      const int s = lane & 15;
      const int kb = ks * 16 + 8 * (lane >> 5);
      const int col = row0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
      const bf16_t* p0 = lds + (kb + (s >> 2)) * (ROWS + PAD) + col;
      const bf16_t* p1 = p0 + 4 * (ROWS + PAD);
      typedef __attribute__((address_space(3))) short4_t* lds_ptr;
      short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
      short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p1));
      short8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8_t, both);
    }
  }

  template <class SrcFn, class Epi>
  __device__ static void run(char* smem, int n_iters, SrcFn src, int64_t lda, int64_t ldb, int m_valid,
                             int n_valid, Epi epi) {
    bf16_t* As = (bf16_t*)smem;
    bf16_t* Bs = As + A_ELEMS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave / WN) * (BM / WM), wn0 = (wave % WN) * (BN / WN);

    f32x16_t acc[NB][TM][TN];
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
          for (int r = 0; r < 16; r++) acc[nb][i][j][r] = 0.f;

    uint4 ra[A_VEC], rb[NB][B_VEC];
    if (n_iters > 0) {
      IterSrc<bf16_t, NB> s = src(0);
      gload<BM, A_VEC, A_KC>(s.a, lda, m_valid, s.k_left, ra);
#pragma unroll
      for (int nb = 0; nb < NB; nb++) gload<BN, B_VEC, B_KC>(s.b[nb], ldb, n_valid, s.k_left, rb[nb]);
    }
    for (int it = 0; it < n_iters; it++) {
      sstore<BM, A_VEC, A_KC>(As, ra);
#pragma unroll
      for (int nb = 0; nb < NB; nb++) sstore<BN, B_VEC, B_KC>(Bs + nb * B_ELEMS, rb[nb]);
      __syncthreads();
      if (it + 1 < n_iters) {  // next tile travels while this one is multiplied
        IterSrc<bf16_t, NB> s = src(it + 1);
        gload<BM, A_VEC, A_KC>(s.a, lda, m_valid, s.k_left, ra);
#pragma unroll
        for (int nb = 0; nb < NB; nb++) gload<BN, B_VEC, B_KC>(s.b[nb], ldb, n_valid, s.k_left, rb[nb]);
      }
#pragma unroll
      for (int ks = 0; ks < BK / 16; ks++) {
        bf16x8_t af[TM], bfr[NB][TN];
#pragma unroll
        for (int i = 0; i < TM; i++) af[i] = frag<BM, A_KC>(As, wm0 + i * 32, ks);
#pragma unroll
        for (int nb = 0; nb < NB; nb++)
#pragma unroll
          for (int j = 0; j < TN; j++) bfr[nb][j] = frag<BN, B_KC>(Bs + nb * B_ELEMS, wn0 + j * 32, ks);
#pragma unroll
        for (int nb = 0; nb < NB; nb++)
#pragma unroll
          for (int i = 0; i < TM; i++)
#pragma unroll
            for (int j = 0; j < TN; j++)
              // operands exchanged: the result register r of lane l is C[m = l%32][n = 8*(r/4) + 4*(l/32) + r%4]
              acc[nb][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[nb][j], af[i], acc[nb][i][j], 0, 0, 0);
      }
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
          float vals[NB][4];
#pragma unroll
          for (int nb = 0; nb < NB; nb++)
#pragma unroll
            for (int q = 0; q < 4; q++) vals[nb][q] = acc[nb][i][j][4 * g + q];
          epi(wm0 + i * 32 + (lane & 31), wn0 + j * 32 + 8 * g + 4 * (lane >> 5), vals);
        }
  }
};

}  // namespace moe
