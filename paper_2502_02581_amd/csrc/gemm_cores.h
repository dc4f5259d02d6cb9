// Tile cores of the grouped GEMMs: an fp32 FMA core (correctness path for MOE_F32) and a
// bf16 MFMA core for gfx950 (v_mfma_f32_32x32x16_bf16, operands staged through LDS).
//
// Both cores compute, for one block, acc[nb][..] = sum over iterations of A_tile * B_tile(nb)
// and hand groups of four consecutive columns to an epilogue functor:
//     epi(m, n, vals)   m, n relative to the block tile;  vals[nb][0..3] = C[m][n..n+3]
// The sum over K runs over n_segs segments of nk iterations each (segments: the shared experts of
// a down projection, the two products of an input gradient); a segment functor supplies where the
// tiles of a segment start, and the cores step along K from there themselves.
#pragma once

#include "moe_common.h"
#include "trace.h"

namespace moe {
// An epilogue functor may read global memory at the position it writes (an activation's saved input,
// an output it accumulates into).  If it says how many 16-byte pieces per position (`kAux`) and offers
// `prefetch(m, n)` returning them, the LDS-DMA core requests the pieces of a whole block of rows
// before it needs them and hands each back through a fourth argument; otherwise the functor does
// its own loads, one position after the other.
template <class E, class = void> struct EpiAux { static constexpr int value = 0; };
template <class E> struct EpiAux<E, std::void_t<decltype(E::kAux)>> { static constexpr int value = E::kAux; };

// Start of one segment.  Pointers are already offset to the tile's first row/column at k = 0;
// "kc" (K-contiguous) operands are [rows][K] row-major, otherwise [K][rows] row-major.
template <typename T, int NB>
struct SegSrc {
  const T* a;        // A tile origin
  const T* b[NB];    // B tile origin(s)
  int k_len;         // values of K in the segment
  // bytes from the origins to the end of the valid data of the tile (used by the cores that load
  // through bounds-checked buffer descriptors: anything at or beyond reads as zero)
  int64_t a_bytes, b_bytes;
};

// Where row m of the A tile lives.  Plain tiles: row m of the tile (the tile origin is part of the
// operand pointers).  Gathered tiles (K-contiguous A only): row idx[row0 + m] / div of the whole
// operand, whose origin the pointers then are -- the token rows of X or dY read in grouped order
// without a permuted copy.
struct RowMap {
  const int32_t* idx;  // NULL: plain
  int32_t div, row0, rows;  // rows: valid rows of the tile (rows at or beyond read as zero)
  __device__ __forceinline__ bool gathered() const { return idx != nullptr; }
  __device__ __forceinline__ int64_t operator()(int m) const { return idx ? (int64_t)(idx[row0 + m] / div) : (int64_t)m; }
};

// What one K iteration reads, for the cores that address element by element.
template <typename T, int NB>
struct IterSrc {
  const T* a;        // A tile origin for this iteration (k offset included)
  const T* b[NB];    // B tile origin(s)
  int k_left;        // valid K elements from this origin on
};
template <typename T, int NB, bool A_KC, bool B_KC, class SegFn>
__device__ __forceinline__ IterSrc<T, NB> iter_src(SegFn& segf, int it, int nk, int BK, int64_t lda, int64_t ldb) {
  const int sg = it / nk, k0 = (it - sg * nk) * BK;
  const SegSrc<T, NB> g = segf(sg);
  IterSrc<T, NB> s;
  s.a = g.a + (A_KC ? (int64_t)k0 : (int64_t)k0 * lda);
#pragma unroll
  for (int nb = 0; nb < NB; nb++) s.b[nb] = g.b[nb] + (B_KC ? (int64_t)k0 : (int64_t)k0 * ldb);
  s.k_left = g.k_len - k0;
  return s;
}

// ------------------------------------------------------------------------------ fp32 core
template <int NB, bool A_KC, bool B_KC>
struct F32Core {
  typedef float T;
  static constexpr int BM = 64, BN = 64, BK = 16, NT = 256;
  static constexpr int LD = 64 + 4;
  static constexpr int LDS_BYTES = (BK * LD + NB * BK * LD) * 4;

  template <class SegFn, class Epi>
  __device__ static void run(char* smem, int n_segs, int nk, SegFn segf, int64_t lda, int64_t ldb, int m_valid,
                             int n_valid, Epi epi, const RowMap& amap) {
    const int n_iters = n_segs * nk;
    auto src = [&](int it) { return iter_src<float, NB, A_KC, B_KC>(segf, it, nk, BK, lda, ldb); };
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
        if (m < m_valid && k < s.k_left) v = A_KC ? s.a[amap(m) * lda + k] : s.a[(int64_t)k * lda + m];
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
template <int BM_, int BN_, int NB, bool A_KC, bool B_KC, int WM_ = 2, int WN_ = 2>
struct MfmaCore {
  typedef bf16_t T;
  static constexpr int BM = BM_, BN = BN_, BK = 64, NT = 256;
  static constexpr int WM = WM_, WN = WN_;
  static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  static constexpr int PAD = 32;
  static constexpr int A_ELEMS = A_KC ? BM * BK : BK * (BM + PAD);
  static constexpr int B_ELEMS = B_KC ? BN * BK : BK * (BN + PAD);
  static constexpr int STAGE_ELEMS = A_ELEMS + NB * B_ELEMS;
  static constexpr int LDS_BYTES = 2 * STAGE_ELEMS * 2;  // two stages
  static constexpr int A_VEC = (BM * BK / 8 + NT - 1) / NT;
  static constexpr int B_VEC = (BN * BK / 8 + NT - 1) / NT;
  static_assert(WM * WN == 4, "four wavefronts per block");
  static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "wave tile must be a multiple of 32");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of a gfx950 CU");

  // ---- global -> registers (16 bytes per access), zero outside the valid extents
  template <int ROWS, int NVEC, bool KC>
  __device__ static __forceinline__ void gload(const bf16_t* base, int64_t ld, int rows_valid, int k_left,
                                               uint4 (&r)[NVEC], const RowMap& map) {
#pragma unroll
    for (int i = 0; i < NVEC; i++) {
      const int v = threadIdx.x + i * NT;
      int row, kk;
      if (KC) { row = v / (BK / 8); kk = (v % (BK / 8)) * 8; }
      else { kk = v / (ROWS / 8); row = (v % (ROWS / 8)) * 8; }
      const bool ok = row < rows_valid && kk < k_left && (ROWS * BK / 8 % NT == 0 || v < ROWS * BK / 8);
      r[i] = make_uint4(0, 0, 0, 0);
      if (ok) {
        const bf16_t* p = KC ? base + (map.gathered() ? map(row) : (int64_t)row) * ld + kk : base + (int64_t)kk * ld + row;
        r[i] = *reinterpret_cast<const uint4*>(p);
      }
    }
  }
  // ---- registers -> LDS
  template <int ROWS, int NVEC, bool KC>
  __device__ static __forceinline__ void sstore(bf16_t* lds, const uint4 (&r)[NVEC]) {
#pragma unroll
    for (int i = 0; i < NVEC; i++) {
      const int v = threadIdx.x + i * NT;
      if (ROWS * BK / 8 % NT != 0 && v >= ROWS * BK / 8) continue;
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
      // transposing read: within 16 lanes, lane s points at 4 consecutive columns of row
      // k = kb + s/4, starting at column 4*(s%4); it receives k = kb..kb+3 of column s.
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

  struct Frags {
    bf16x8_t a[TM], b[NB][TN];
  };
  __device__ static __forceinline__ void load_frags(const bf16_t* As, const bf16_t* Bs, int wm0, int wn0, int ks,
                                                    Frags& f) {
#pragma unroll
    for (int i = 0; i < TM; i++) f.a[i] = frag<BM, A_KC>(As, wm0 + i * 32, ks);
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
      for (int j = 0; j < TN; j++) f.b[nb][j] = frag<BN, B_KC>(Bs + nb * B_ELEMS, wn0 + j * 32, ks);
  }
  __device__ static __forceinline__ void mma(f32x16_t (&acc)[NB][TM][TN], const Frags& f) {
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          // operands exchanged: result register r of lane l is C[m = l%32][n = 8*(r/4) + 4*(l/32) + r%4]
          acc[nb][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[nb][j], f.a[i], acc[nb][i][j], 0, 0, 0);
  }

  template <class SegFn, class Epi>
  __device__ static void run(char* smem, int n_segs, int nk, SegFn segf, int64_t lda, int64_t ldb, int m_valid,
                             int n_valid, Epi epi, const RowMap& amap) {
    const int n_iters = n_segs * nk;
    auto src = [&](int it) { return iter_src<bf16_t, NB, A_KC, B_KC>(segf, it, nk, BK, lda, ldb); };
    const RowMap plain = {nullptr, 1, 0, 0};
    bf16_t* lds = (bf16_t*)smem;
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
    auto fetch = [&](int it) {
      IterSrc<bf16_t, NB> s = src(it);
      gload<BM, A_VEC, A_KC>(s.a, lda, m_valid, s.k_left, ra, amap);
#pragma unroll
      for (int nb = 0; nb < NB; nb++) gload<BN, B_VEC, B_KC>(s.b[nb], ldb, n_valid, s.k_left, rb[nb], plain);
    };
    auto stash = [&](int stage) {
      bf16_t* As = lds + stage * STAGE_ELEMS;
      sstore<BM, A_VEC, A_KC>(As, ra);
#pragma unroll
      for (int nb = 0; nb < NB; nb++) sstore<BN, B_VEC, B_KC>(As + A_ELEMS + nb * B_ELEMS, rb[nb]);
    };

    if (n_iters > 0) {
      fetch(0);
      stash(0);
      if (n_iters > 1) fetch(1);
      __syncthreads();
    }
    Frags f0, f1;
    if (n_iters > 0) load_frags(lds, lds + A_ELEMS, wm0, wn0, 0, f0);
    for (int it = 0; it < n_iters; it++) {
      const bf16_t* As = lds + (it & 1) * STAGE_ELEMS;
      const bf16_t* Bs = As + A_ELEMS;
      load_frags(As, Bs, wm0, wn0, 1, f1);
      mma(acc, f0);
      // the tile of iteration it+1 (in registers since the previous iteration) goes to the other
      // stage; the tile of iteration it+2 starts its trip from HBM/L2
      if (it + 1 < n_iters) stash((it + 1) & 1);
      if (it + 2 < n_iters) fetch(it + 2);
      load_frags(As, Bs, wm0, wn0, 2, f0);
      mma(acc, f1);
      load_frags(As, Bs, wm0, wn0, 3, f1);
      mma(acc, f0);
      mma(acc, f1);
      __syncthreads();
      if (it + 1 < n_iters) {
        const bf16_t* An = lds + ((it + 1) & 1) * STAGE_ELEMS;
        load_frags(An, An + A_ELEMS, wm0, wn0, 0, f0);
      }
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

// ------------------------------------------------------------------ bf16 MFMA core, LDS DMA loads
// Same math as MfmaCore, but tiles travel HBM/L2 -> LDS directly (buffer_load_dwordx4 ... lds),
// so no registers stage them.  Lane l of a wave-wide load lands at lds_base + 16*l, which fixes
// each tile to whole 1 KB pieces per instruction; the swizzles are applied on the global side
// (which 16-byte piece a lane fetches).  Out-of-range pieces read as zero through the buffer
// descriptor's num_records, which provides the zero fill of ragged row and K tails.
// Requires K-contiguous operands to have K % 64 == 0 (a K tail inside a row cannot be masked).
//
// LDS layouts (bf16 elements), BK = 64, no padding:
//  K-contiguous operand [rows][64]: 16-byte piece c of a row sits at position c ^ ((row/2)%8), so
//    that the 16 rows one phase of a 16-byte-per-lane read touches cover all banks once.
//  row-contiguous operand [64 k][ROWS]: piece c (8 columns) of k-row k sits at position
//    c ^ (4*(k%4)), which spreads the four k rows of a transposing read over all banks.
template <int BM_, int BN_, int NB, bool A_KC, bool B_KC, int WM_ = 2, int WN_ = 2, int DEPTH = 1>
struct MfmaDmaCore {
  typedef bf16_t T;
  static constexpr int BM = BM_, BN = BN_, BK = 64;
  static constexpr int KS = BK / 16;  // MFMA k-steps per tile slot
  static constexpr int WM = WM_, WN = WN_;
  static constexpr int NW = WM * WN, NT = 64 * NW;  // wavefronts and threads per block
  static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  static constexpr int A_ELEMS = BM * BK, B_ELEMS = BN * BK;
  // Software pipeline of the K loop, by DEPTH:
  //  1  (tall tiles, bound by the matrix pipe): a ring of three A tiles and a ring of two B tile
  //     sets.  The A tile of iteration t+2 is requested while the B tiles of t+1 are still
  //     landing, so the memory pipeline never runs dry at the per-iteration barrier; MFMAs, LDS
  //     reads and tile loads are interleaved by hand.
  //  >= 2  (short tiles of ragged groups, bound by streaming the other operand from HBM): DEPTH + 1
  //     slots per operand and the loads of iteration t + DEPTH issued in iteration t, so that DEPTH
  //     whole K steps are in flight per CU; the latency of an HBM stream, not the matrix pipe, sets
  //     the pace there.
  //  0  (weight gradients of groups with a handful of rows: K is one or two steps): one slot, no
  //     pipeline, small enough in LDS and registers for several blocks per CU, which is what hides
  //     latency when a block's life is one K iteration and an epilogue.
  static constexpr bool RING = DEPTH == 1;
  static constexpr int A_SLOTS = DEPTH == 0 ? 1 : DEPTH == 1 ? 3 : DEPTH + 1;
  static constexpr int B_SLOTS = DEPTH == 0 ? 1 : DEPTH == 1 ? 2 : DEPTH + 1;
  static constexpr int B_SET_ELEMS = NB * B_ELEMS;
  static constexpr int TILE_BYTES = (A_SLOTS * A_ELEMS + B_SLOTS * B_SET_ELEMS) * 2;
  static constexpr int STAGING_BYTES = NW * NB * 32 * ((BN_ / WN_) + 4) * 4;  // epilogue, see run()
  static constexpr int LDS_BYTES = TILE_BYTES > STAGING_BYTES ? TILE_BYTES : STAGING_BYTES;
  static constexpr int A_NI = BM * BK / (512 * NW), B_NI = BN * BK / (512 * NW);  // wave-wide loads per wave and tile
  static constexpr int PR_KC = BK / 8;  // 16-byte pieces per row of a K-contiguous tile
  static_assert(NW == 4 || NW == 8, "four or eight wavefronts per block");
  static_assert(BM * BK % (512 * NW) == 0 && BN * BK % (512 * NW) == 0,
                "every wave issues the same number of 1 KB loads per tile");
  static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "wave tile must be a multiple of 32");
  static_assert((A_KC || BM % 128 == 0) && (B_KC || BN % 128 == 0),
                "swizzle of row-contiguous tiles needs >= 16 pieces per k row");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of a gfx950 CU");
  typedef __attribute__((address_space(3))) void* lds_vptr;

  // Byte offset (from the tile origin in memory) of the piece that lane `lane` of wave `wave`
  // fetches with its FIRST load.  The j-th load of the same lane is j * load_stride() rows further
  // on (the swizzle terms do not depend on j); run() keeps one offset register per load, so that
  // the K loop spends no instructions on addresses and the whole offset stays inside the
  // descriptor's bounds check.
  __device__ static __forceinline__ int kc_swizzle(int row) { return ((row * PR_KC) >> 4) & (PR_KC - 1); }
  template <int ROWS, bool KC>
  __device__ static __forceinline__ uint32_t piece_offset(int wave, int lane, uint32_t ld) {
    const int q = wave * 64 + lane;  // linear 16-byte piece of the LDS tile
    if (KC) {
      const int row = q / PR_KC, pos = q % PR_KC;
      const int c = pos ^ kc_swizzle(row);
      return (uint32_t)row * ld * 2u + (uint32_t)c * 16u;
    } else {
      constexpr int PR = ROWS / 8;
      const int k = q / PR, pos = q % PR;
      const int c = pos ^ (4 * (k & 3));
      return (uint32_t)k * ld * 2u + (uint32_t)c * 16u;
    }
  }
  // rows of the memory operand (K-contiguous: tile rows; row-contiguous: k rows) between two
  // consecutive loads of a wave: NW waves x 1 KB of LDS tile per round
  template <int ROWS, bool KC>
  __device__ static constexpr int load_stride() { return KC ? 512 * NW / BK : 512 * NW / ROWS; }

  // One wave-wide 16-byte-per-lane load straight into LDS: the n-th 1 KB piece of this wave's share
  // of a tile.  Written as inline assembly so that the compiler does not serialise it against the
  // LDS reads of the other stage (it would wait for vmcnt(0) before every ds_read that may alias);
  // run() waits for the loads itself before its barrier.
  typedef __attribute__((ext_vector_type(4))) int rsrc_t;
  // `rsrc` is the raw buffer descriptor of the tile (48-bit base, stride 0, byte count, 32-bit data
  // format), `voff` the lane's byte offset from its base (piece_offset plus the rows of the earlier
  // loads of the tile), `dst` the LDS byte address of this wave's 1 KB piece.
  //
  // The compiler's hazard recogniser does not look inside inline assembly.  M0 must not be read by an
  // LDS-DMA load in the wait state after its write, hence the s_nop.  The descriptor words must not
  // have been written by a VALU instruction (v_readfirstlane and the like) in the five wait states
  // before the load: they are kept in scalar registers and stepped with scalar instructions only
  // (see Cursor), far from any vector instruction that could produce them.
  __device__ static __forceinline__ void issue_one(const rsrc_t& rsrc, uint32_t dst, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(dst), "v"(voff), "s"(rsrc)
                 : "memory");
  }

  // ---- LDS -> MFMA fragment: lane l holds k = 16*ks + 8*(l/32) + 0..7 of row (row0 + l%32).
  // All lane-dependent address arithmetic is done once (lane_offsets); inside the K loop a
  // fragment address is a per-lane base plus a compile-time constant, which the LDS instructions
  // carry in their offset field.
  //   K-contiguous tile:   off[ks] for the wave's first 32 rows; 32 more rows = +32*BK elements
  //                        (the swizzle repeats every 16 rows)
  //   row-contiguous tile: off[t] for the t-th group of 32 columns at k-step 0;
  //                        k-step ks = +16*ks*ROWS elements, second half of the 8 k = +4*ROWS
  template <int ROWS, bool KC, int NTILE>
  __device__ static __forceinline__ void lane_offsets(int w0, int lane, int (&off)[4]) {
    if (KC) {
      const int row = w0 + (lane & 31);
#pragma unroll
      for (int ks = 0; ks < KS; ks++) off[ks] = row * BK + (((ks * 2 + (lane >> 5)) ^ kc_swizzle(row)) << 3);
    } else {
      // transposing read: within 16 lanes, lane s points at 4 consecutive columns of k-row
      // kb + s/4, starting at column 4*(s%4); it receives k = kb..kb+3 of column s.
      const int s = lane & 15;
      const int k = 8 * (lane >> 5) + (s >> 2);
#pragma unroll
      for (int t = 0; t < 4; t++) {
        const int col = w0 + t * 32 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
        off[t] = k * ROWS + (((col >> 3) ^ (4 * (k & 3))) << 3) + (col & 7);
      }
    }
  }
  template <int ROWS, bool KC>
  __device__ static __forceinline__ bf16x8_t frag(const bf16_t* tile, const int (&off)[4], int t, int ks) {
    if (KC) {
      const uint4 v = *reinterpret_cast<const uint4*>(tile + off[ks] + t * 32 * BK);
      return __builtin_bit_cast(bf16x8_t, v);
    } else {
      typedef __attribute__((address_space(3))) short4_t* lds_ptr;
      const bf16_t* p0 = tile + off[t] + ks * 16 * ROWS;
      short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
      short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0 + 4 * ROWS));
      short8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8_t, both);
    }
  }

  struct Frags {
    bf16x8_t a[TM], b[NB][TN];
  };
  // the r-th fragment load of a k-step: first the TM fragments of A, then the NB*TN of B
  static constexpr int kFragLoads = TM + NB * TN;
  __device__ static __forceinline__ void load_frag_n(const bf16_t* As, const bf16_t* Bs, const int (&ao)[4],
                                                     const int (&bo)[4], int ks, int r, Frags& f) {
    if (r < TM) {
      f.a[r] = frag<BM, A_KC>(As, ao, r, ks);
    } else {
      const int nb = (r - TM) / TN, j = (r - TM) % TN;
      f.b[nb][j] = frag<BN, B_KC>(Bs + nb * B_ELEMS, bo, j, ks);
    }
  }
  // MFMA number m of a k-step.  Inline assembly with a memory clobber: the instruction stream of
  // the K loop is then exactly the order written in run() (LDS reads, tile loads and MFMAs
  // interleaved by hand), the compiler only allocates registers and inserts the waits.
  // Operands exchanged: result register r of lane l is C[m = l%32][n = 8*(r/4) + 4*(l/32) + r%4].
  static constexpr int kMfma = NB * TM * TN;
  __device__ static __forceinline__ void mfma_n(f32x16_t (&acc)[NB][TM][TN], const Frags& f, int m) {
    const int nb = m / (TM * TN), i = (m / TN) % TM, j = m % TN;
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
                 : "+a"(acc[nb][i][j])
                 : "v"(f.b[nb][j]), "v"(f.a[i])
                 : "memory");
  }

  // Position of a stream of tile loads along K.  The K loop pays for every scalar instruction between
  // its MFMAs, so stepping is a handful of additions; the segment functor is consulted only where a
  // segment starts.  Once the product is exhausted the steps are zero and the byte counts stay at
  // zero: loads issued from there on read nothing and deliver zeros.
  struct Cursor {
    rsrc_t ad, bd[NB];      // buffer descriptors of the A tile and the B tile(s) at this position
    int64_t a_rem, b_rem;   // bytes from the tile origins to the end of the tile's valid data
    int64_t a_step, b_step; // bytes by which one iteration moves the origins
    int k_left, k_step;     // valid values of K from the origins on
    int ki, sg;
  };
  // byte count of a descriptor: 32 bits, saturating (built from the halves: scalar instructions only)
  __device__ static __forceinline__ int clip_rem(int64_t v) {
    const int32_t hi = (int32_t)(v >> 32);
    return hi < 0 ? 0 : hi > 0 ? -1 : (int)(uint32_t)v;
  }
  __device__ static __forceinline__ rsrc_t make_desc(const bf16_t* base, int64_t bytes) {
    const uint64_t p = (uint64_t)base;
    rsrc_t r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)p);
    r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(p >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane(clip_rem(bytes));
    r[3] = 0x00020000;
    return r;
  }
  // moves a descriptor's base by `step` bytes (the base stays below 2^48) and sets its byte count
  __device__ static __forceinline__ void move_desc(rsrc_t& r, int64_t step, int64_t bytes) {
    const uint64_t p = (((uint64_t)(uint32_t)r[1] << 32) | (uint32_t)r[0]) + (uint64_t)step;
    r[0] = (int)(uint32_t)p;
    r[1] = (int)(uint32_t)(p >> 32);
    r[2] = clip_rem(bytes);
  }
  template <class SegFn>
  __device__ static __forceinline__ void seek(Cursor& c, SegFn& segf, int sg, int n_segs, int nk, int64_t lda,
                                              int64_t ldb) {
    c.ki = 0;
    c.sg = sg;
    if (sg < n_segs && nk > 0) {
      const SegSrc<bf16_t, NB> g = segf(sg);
      c.a_rem = g.a_bytes;
      c.b_rem = g.b_bytes;
      c.ad = make_desc(g.a, c.a_rem);
#pragma unroll
      for (int nb = 0; nb < NB; nb++) c.bd[nb] = make_desc(g.b[nb], c.b_rem);
      // The words above come out of v_readfirstlane.  Five wait states must pass before a tile load reads
      // them, wherever the compiler places that load (a segment starts once or twice per tile, so this
      // costs nothing); the statements are tied to the descriptors and keep their order, so the wait
      // stands behind the last of those writes.
#pragma unroll
      for (int nb = 0; nb < NB; nb++) asm volatile("" : "+s"(c.bd[nb]) : : "memory");
      asm volatile("s_nop 4" : "+s"(c.ad) : : "memory");
      c.a_step = A_KC ? (int64_t)BK * 2 : (int64_t)BK * 2 * lda;
      c.b_step = B_KC ? (int64_t)BK * 2 : (int64_t)BK * 2 * ldb;
      c.k_left = g.k_len;
      c.k_step = BK;
    } else {
      // exhausted (or nothing to do): zero-length descriptors that stay where they are
      c.a_rem = c.b_rem = c.a_step = c.b_step = 0;
      c.k_left = c.k_step = 0;
      if (sg == 0) {
        c.ad = make_desc(nullptr, 0);
#pragma unroll
        for (int nb = 0; nb < NB; nb++) c.bd[nb] = make_desc(nullptr, 0);
      } else {
        c.ad[2] = 0;
#pragma unroll
        for (int nb = 0; nb < NB; nb++) c.bd[nb][2] = 0;
      }
    }
  }
  template <class SegFn>
  __device__ static __forceinline__ void next(Cursor& c, SegFn& segf, int n_segs, int nk, int64_t lda, int64_t ldb) {
    c.ki++;
    if (c.ki != nk) {
      c.a_rem -= c.a_step;
      c.b_rem -= c.b_step;
      move_desc(c.ad, c.a_step, c.a_rem);
#pragma unroll
      for (int nb = 0; nb < NB; nb++) move_desc(c.bd[nb], c.b_step, c.b_rem);
      c.k_left -= c.k_step;
    } else {
      seek(c, segf, c.sg + 1, n_segs, nk, lda, ldb);
    }
  }

  template <class SegFn, class Epi>
  // (the valid extents are not needed here: the descriptors' byte counts zero-fill the loads and the
  // epilogue functor masks the stores)
  __device__ static __forceinline__ void run(char* smem, int n_segs, int nk, SegFn segf, int64_t lda, int64_t ldb,
                                             int /*m_valid*/, int /*n_valid*/, Epi epi, const RowMap& amap) {
    const int n_iters = n_segs * nk;
    MOE_PHASE(0);
    bf16_t* lds = (bf16_t*)smem;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm0 = (wave / WN) * (BM / WM), wn0 = (wave % WN) * (BN / WN);

    f32x16_t acc[NB][TM][TN];
    // Called once the first tile loads are on their way, so that the 16 * NB * TM * TN register
    // writes overlap their latency.
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
          for (int j = 0; j < TN; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[nb][i][j][r] = 0.f;
      // Pin the zeroing here.  Left alone, the compiler may materialise an accumulator's zeros right
      // in front of its first MFMA; that MFMA is inline assembly, so nobody would insert the wait
      // states a VALU write to an accumulator register needs before an MFMA reads it.
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
          for (int j = 0; j < TN; j++) asm volatile("" : "+a"(acc[nb][i][j])::"memory");
      asm volatile("s_nop 7" ::: "memory");
    };

    // per-lane byte offsets of this wave's loads of a tile, fixed for the whole K loop
    uint32_t voa[A_NI], vob[B_NI];
#pragma unroll
    for (int j = 0; j < A_NI; j++)
      voa[j] = piece_offset<BM, A_KC>(wave, lane, (uint32_t)lda) + (uint32_t)(j * load_stride<BM, A_KC>()) * (uint32_t)lda * 2u;
    if constexpr (A_KC) {
      // gathered A rows: the same pieces, from the rows the map names.  The descriptor then spans the
      // whole operand, so the rows beyond the tile's valid ones get an offset no descriptor reaches
      // (they read as zero, as they do past the end of a plain tile).
      if (amap.gathered()) {
        const int q = wave * 64 + lane, row = q / PR_KC, c = (q % PR_KC) ^ kc_swizzle(row);
#pragma unroll
        for (int j = 0; j < A_NI; j++) {
          const int r = row + j * load_stride<BM, A_KC>();
          voa[j] = r < amap.rows ? (uint32_t)amap(r) * (uint32_t)lda * 2u + (uint32_t)c * 16u : 0xffffff00u;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < B_NI; j++)
      vob[j] = piece_offset<BN, B_KC>(wave, lane, (uint32_t)ldb) + (uint32_t)(j * load_stride<BN, B_KC>()) * (uint32_t)ldb * 2u;
    // LDS byte addresses: this wave's first piece of A slot 0 and of B slot 0
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t lds_a0 = lds_addr + (uint32_t)wave * 1024u;
    const uint32_t lds_b0 = lds_a0 + (uint32_t)(A_SLOTS * A_ELEMS * 2);
    auto load_a = [&](const Cursor& c, int slot, int j) __attribute__((always_inline)) {
      issue_one(c.ad, lds_a0 + (uint32_t)(slot * A_ELEMS * 2) + (uint32_t)(j * NW) * 1024u, voa[j]);
    };
    auto load_b = [&](const Cursor& c, int slot, int n) __attribute__((always_inline)) {
      const int nb = n / B_NI, j = n % B_NI;
      issue_one(c.bd[nb], lds_b0 + (uint32_t)((slot * B_SET_ELEMS + nb * B_ELEMS) * 2) + (uint32_t)(j * NW) * 1024u, vob[j]);
    };
    // Loads beyond the last iteration still issue (the wait counts below stay constant and the K
    // loop free of branches): an exhausted cursor makes them read nothing.
    auto start = [&](Cursor& c) __attribute__((always_inline)) { seek(c, segf, 0, n_segs, nk, lda, ldb); };
    auto step = [&](Cursor& c) __attribute__((always_inline)) { next(c, segf, n_segs, nk, lda, ldb); };

    static_assert(TM <= 4 && TN <= 4, "lane_offsets holds four tiles per operand");
    int ao[4], bo[4];
    lane_offsets<BM, A_KC, TM>(wm0, lane, ao);
    lane_offsets<BN, B_KC, TN>(wn0, lane, bo);

    constexpr int kLoadsB = NB * B_NI;  // loads per wave for the B tiles of one iteration
    if constexpr (DEPTH >= 2) {
      // streaming pipeline: tiles t .. t+DEPTH-1 in flight while tile t is multiplied
      constexpr int L = A_NI + kLoadsB;  // loads per wave and iteration
      static_assert((DEPTH - 1) * L <= 63, "the wait count of the oldest tile must be encodable");
      Cursor s0;  // the next tile to request
      start(s0);
      auto issue_tile = [&](int it) __attribute__((always_inline)) {
        const int slot = it % (DEPTH + 1);
#pragma unroll
        for (int j = 0; j < A_NI; j++) load_a(s0, slot, j);
#pragma unroll
        for (int n = 0; n < kLoadsB; n++) load_b(s0, slot, n);
        step(s0);
      };
      if (n_iters > 0) {
        for (int it = 0; it < DEPTH; it++) issue_tile(it);
      }
      zero_acc();
      for (int it = 0; it < n_iters; it++) {
        // tile `it` has landed once at most the DEPTH - 1 younger tiles are outstanding (loads
        // complete in order); the barrier also says that every wave is done with tile it - 1,
        // whose slot the loads of tile it + DEPTH overwrite
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DEPTH - 1) * L) : "memory");
        __syncthreads();
        issue_tile(it + DEPTH);
        const int slot = it % (DEPTH + 1);
        const bf16_t* As = lds + slot * A_ELEMS;
        const bf16_t* Bs = lds + A_SLOTS * A_ELEMS + slot * B_SET_ELEMS;
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
          Frags f;
#pragma unroll
          for (int r = 0; r < kFragLoads; r++) load_frag_n(As, Bs, ao, bo, ks, r, f);
#pragma unroll
          for (int m = 0; m < kMfma; m++) mfma_n(acc, f, m);
        }
      }
    } else if constexpr (!RING) {
      // single slot: load a tile, wait, multiply; k-steps beyond the rows of K are skipped
      Cursor s0;
      start(s0);
      zero_acc();
      for (int it = 0; it < n_iters; it++) {
        if (it > 0) __syncthreads();
#pragma unroll
        for (int j = 0; j < A_NI; j++) load_a(s0, 0, j);
#pragma unroll
        for (int n = 0; n < kLoadsB; n++) load_b(s0, 0, n);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
          if (ks * 16 >= s0.k_left) continue;  // uniform: the remaining k rows of the tile are zero
          Frags f;
#pragma unroll
          for (int r = 0; r < kFragLoads; r++) load_frag_n(lds, lds + A_SLOTS * A_ELEMS, ao, bo, ks, r, f);
#pragma unroll
          for (int m = 0; m < kMfma; m++) mfma_n(acc, f, m);
        }
        step(s0);
      }
    } else {
    Cursor s1, s2;  // s1: the B tiles of iteration it + 1; s2: the A tile of iteration it + 2
    start(s1);
    start(s2);
    if (n_iters > 0) {
#pragma unroll
      for (int j = 0; j < A_NI; j++) load_a(s2, 0, j);
#pragma unroll
      for (int n = 0; n < kLoadsB; n++) load_b(s1, 0, n);
      step(s1);
      step(s2);
#pragma unroll
      for (int j = 0; j < A_NI; j++) load_a(s2, 1, j);
      step(s2);
    }
    zero_acc();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    MOE_PHASE(1);

    // A wave issues in order and a tile load holds it for as long as the memory pipeline has no
    // free slot, so the overlap of loads, LDS reads and MFMAs is written into the instruction
    // stream itself.  Per K iteration t (4 k-steps
    // of kMfma MFMAs):
    //   - the fragments of k-step ks+1 are read from LDS during the MFMAs of ks, one per MFMA;
    //   - the loads of B(t+1), then of A(t+2), are spread evenly between the MFMAs;
    //   - half-way through the last k-step all LDS reads of this iteration are done: wait until
    //     B(t+1) has landed (A(t+2) may still be in flight: loads complete in order), barrier, and
    //     read the first fragments of iteration t+1 under the remaining MFMAs.
    constexpr int kLoads = kLoadsB + A_NI;
    constexpr int kHalf = kMfma / 2;                 // MFMAs of the last k-step before the barrier
    constexpr int kSlots = (KS - 1) * kMfma + kHalf; // MFMA slots before the barrier: all loads issue here
    constexpr int kLate = kMfma - kHalf;             // MFMAs after the barrier
    Frags f[2];
#pragma unroll
    for (int r = 0; r < kFragLoads; r++) load_frag_n(lds, lds + A_SLOTS * A_ELEMS, ao, bo, 0, r, f[0]);
    int a_cur = 0, b_cur = 0;  // slots of this iteration's tiles
    for (int it = 0; it < n_iters; it++) {
      const int a_nxt = a_cur == A_SLOTS - 1 ? 0 : a_cur + 1;   // A(t+1)
      const int a_nn = a_nxt == A_SLOTS - 1 ? 0 : a_nxt + 1;    // A(t+2) goes here
      const int b_nxt = b_cur ^ 1;
      const bf16_t* As = lds + a_cur * A_ELEMS;
      const bf16_t* Bs = lds + A_SLOTS * A_ELEMS + b_cur * B_SET_ELEMS;
      const bf16_t* An = lds + a_nxt * A_ELEMS;
      const bf16_t* Bn = lds + A_SLOTS * A_ELEMS + b_nxt * B_SET_ELEMS;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
#pragma unroll
        for (int m = 0; m < kMfma; m++) {
          if (ks < KS - 1) {
            // fragment loads of k-step ks+1, spread over the MFMAs of ks
#pragma unroll
            for (int r = m * kFragLoads / kMfma; r < (m + 1) * kFragLoads / kMfma; r++)
              load_frag_n(As, Bs, ao, bo, ks + 1, r, f[(ks + 1) & 1]);
          } else {
            if (m == kHalf) {
              // B(t+1) must have landed (the A_NI loads of A(t+2) issued after it may still be
              // outstanding), and every wave must be done reading this iteration's tiles
              asm volatile("s_waitcnt vmcnt(%0)" ::"n"(A_NI) : "memory");
              __syncthreads();
            }
            // first fragments of iteration t+1 under the remaining MFMAs
            // (after the last tile this reads stale but in-bounds LDS data that is never used)
            if (m >= kHalf) {
#pragma unroll
              for (int r = (m - kHalf) * kFragLoads / kLate; r < (m - kHalf + 1) * kFragLoads / kLate; r++)
                load_frag_n(An, Bn, ao, bo, 0, r, f[0]);
            }
          }
          const int slot = ks * kMfma + m;
          if (slot < kSlots) {
#pragma unroll
            for (int n = slot * kLoads / kSlots; n < (slot + 1) * kLoads / kSlots; n++) {
              if (n < kLoadsB) load_b(s1, b_nxt, n);
              else load_a(s2, a_nn, n - kLoadsB);
            }
          }
          mfma_n(acc, f[ks & 1], m);
        }
      }
      step(s1);
      step(s2);
      a_cur = a_nxt;
      b_cur = b_nxt;
    }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // zero-length loads of the tail
    MOE_PHASE(2);
    // The accumulators live in AGPRs.  Each value is copied out right where it is needed (the
    // volatile asm pins the order); left to itself the compiler copies all 256 at the loop exit,
    // needs every arch VGPR for that and spills the loop's address registers.
    // The MFMAs above are opaque to the compiler's hazard recogniser, so the wait between the last
    // MFMA (8 passes of 4 cycles, plus write-back) and the first read of any accumulator is
    // explicit: 6 x 16 idle cycles, attached to the accumulator of the last MFMA.  The empty
    // statements make every other accumulator depend on a point after that wait (volatile asm
    // statements keep their order), so no compiler-generated accumulator copy can move above it.
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15"
                 : "+a"(acc[NB - 1][TM - 1][TN - 1])
                 :
                 : "memory");
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++) asm volatile("" : "+a"(acc[nb][i][j])::"memory");
    // Epilogue through LDS.  In the MFMA result layout a lane owns four consecutive columns of one
    // row, which would make every global store a scatter of 8-byte pieces over 32 rows.  Each wave
    // therefore passes its 32-row blocks through a private LDS region (fp32, rows padded by 16
    // bytes: conflict-free 16-byte writes and reads) and picks them up again with eight
    // consecutive columns per lane, so that the epilogue stores whole 128-byte lines.
    __syncthreads();  // every wave is done with the tile slots (stale fragment reads included)
    constexpr int CW = TN * 32;          // columns of the wave tile (per product)
    constexpr int RS = CW + 4;           // row stride of the staging region, in floats
    constexpr int LPR = CW / 8;          // lanes per row when reading back
    constexpr int RPP = 64 / LPR;        // rows per read pass
    static_assert(NW * NB * 32 * RS * 4 <= LDS_BYTES, "staging regions of the waves fit into LDS");
    static_assert(NW * NB * 32 * RS * 4 == STAGING_BYTES, "STAGING_BYTES matches the staging layout");
    float* stage = reinterpret_cast<float*>(smem) + wave * (NB * 32 * RS);
    constexpr int kAux = EpiAux<Epi>::value;
    constexpr int NPASS = 32 / RPP;
    auto stage_block = [&](int i) __attribute__((always_inline)) {
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
          for (int g = 0; g < 4; g++) {
            float4 v;
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v.x) : "a"(acc[nb][i][j][4 * g + 0]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v.y) : "a"(acc[nb][i][j][4 * g + 1]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v.z) : "a"(acc[nb][i][j][4 * g + 2]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v.w) : "a"(acc[nb][i][j][4 * g + 3]));
            *reinterpret_cast<float4*>(stage + (nb * 32 + (lane & 31)) * RS + j * 32 + 8 * g + 4 * (lane >> 5)) = v;
          }
    };
    auto read_pass = [&](int pass, float (&vals)[NB][8]) __attribute__((always_inline)) {
      const int row = pass * RPP + lane / LPR, c0 = (lane % LPR) * 8;
#pragma unroll
      for (int nb = 0; nb < NB; nb++) {
        const float4 lo = *reinterpret_cast<const float4*>(stage + (nb * 32 + row) * RS + c0);
        const float4 hi = *reinterpret_cast<const float4*>(stage + (nb * 32 + row) * RS + c0 + 4);
        vals[nb][0] = lo.x; vals[nb][1] = lo.y; vals[nb][2] = lo.z; vals[nb][3] = lo.w;
        vals[nb][4] = hi.x; vals[nb][5] = hi.y; vals[nb][6] = hi.z; vals[nb][7] = hi.w;
      }
    };
    const int c0 = (lane % LPR) * 8;
    if constexpr (kAux > 0) {
      // the functor's own global reads of block i + 1 are in flight while block i is staged,
      // converted and stored (everything unrolled: the pieces live in registers)
      typedef decltype(epi.prefetch(0, 0)) Aux;
      Aux aux[2][NPASS];
#pragma unroll
      for (int pass = 0; pass < NPASS; pass++) aux[0][pass] = epi.prefetch(wm0 + pass * RPP + lane / LPR, wn0 + c0);
#pragma unroll
      for (int i = 0; i < TM; i++) {
        stage_block(i);
        if (i + 1 < TM) {
#pragma unroll
          for (int pass = 0; pass < NPASS; pass++)
            aux[(i + 1) & 1][pass] = epi.prefetch(wm0 + (i + 1) * 32 + pass * RPP + lane / LPR, wn0 + c0);
        }
#pragma unroll
        for (int pass = 0; pass < NPASS; pass++) {
          float vals[NB][8];
          read_pass(pass, vals);
          epi(wm0 + i * 32 + pass * RPP + lane / LPR, wn0 + c0, vals, aux[i & 1][pass]);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < TM; i++) {
        stage_block(i);
        // not unrolled: the epilogue functor may be large (activation functions), and a body that is
        // too big keeps the compiler from unrolling the loop over i, which would put the accumulators
        // into scratch memory (their indices must be compile-time constants)
#pragma unroll 1
        for (int pass = 0; pass < NPASS; pass++) {
          float vals[NB][8];
          read_pass(pass, vals);
          epi(wm0 + i * 32 + pass * RPP + lane / LPR, wn0 + c0, vals);
        }
      }
    }
    MOE_PHASE(3);
  }
};

}  // namespace moe
