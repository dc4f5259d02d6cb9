// Tile plan and argument blocks of the grouped GEMMs (device side).
#pragma once

#include "moe_common.h"

namespace moe {

// One row tile of a grouped GEMM whose C rows are token rows.
struct RowTile {
  int32_t group;     // expert that owns the rows
  int32_t row0_in;   // first row in the [n_rows, .] input/output of the call
  int32_t rows;      // valid rows (<= tile height) in bits 0..15, tile kind in bits 16..17
  int32_t row0_out;  // first row in the per-group saved activations (differs in shared mode)
};

__host__ __device__ inline int tile_rows(const RowTile& t) { return t.rows & 0xffff; }
__host__ __device__ inline int tile_kind(const RowTile& t) { return (t.rows >> 16) & 3; }
// heights of the tile kinds of the mixed-height plan (kind 0 is the full tile)
__host__ __device__ inline int kind_height(int kind) { return 256 >> kind; }
// row tiles per band of the XCD-aware tile order of the LDS-DMA path
constexpr int kBandRows = 4;

// Device-built plan, laid out in the workspace.
struct Plan {
  RowTile* tiles;      // [max_tiles]
  int32_t* n_tiles;    // [1]
  int4* ginfo;         // [n_groups] {group, rows, first row, compact slot} by descending row count
};

inline size_t plan_bytes(int n_groups, int max_tiles) {
  return align_up((size_t)max_tiles * sizeof(RowTile), 256) + 256 + align_up((size_t)n_groups * sizeof(int4), 256);
}

inline Plan carve_plan(void* ws, int /*n_groups*/, int max_tiles) {
  char* p = (char*)ws;
  Plan pl;
  pl.tiles = (RowTile*)p;
  p += align_up((size_t)max_tiles * sizeof(RowTile), 256);
  pl.n_tiles = (int32_t*)p;
  p += 256;
  pl.ginfo = (int4*)p;
  return pl;
}

// C[rows, N] (+ second C when dual) = sum over (pair, seg) of A_seg[rows, K] * B_seg[K, N]
struct RowGemm {
  const RowTile* tiles;     // NULL: direct tiling of n_rows rows, single group 0
  const int32_t* n_tiles;
  int32_t n_rows;
  int32_t direct_kind;      // tiles == NULL on the LDS-DMA path: tile kind (height 256 >> kind) of the direct tiling
  int32_t N, K;
  int32_t n_pairs, n_segs;
  const void* A[2];         // per pair; element (row, k) at A + seg*a_seg + row*lda + k
  int64_t lda, a_seg;
  int32_t a_rows_out;       // A rows are indexed by row0_out (saved activations) instead of row0_in
  // gathered A (pair 0, single segment, K-contiguous A only): row r of the call reads row
  // a_index[r] / a_index_div of A, which has a_src_rows rows (NULL: A is indexed by r itself)
  const int32_t* a_index;
  int32_t a_index_div, a_src_rows;
  const void* B[2];         // per pair; + group*b_group + seg*b_seg
  const void* Bdual;        // second B of a dual GEMM (pair 0 only)
  int64_t ldb, b_group, b_seg;
  // epilogue
  void* out[3];
  const void* in[2];
  // activation-backward epilogues: row r of the product is scaled by c_scale[a_index[r]] first (NULL: 1)
  const float* c_scale;
  int64_t ldc;
  int32_t c_rows_out;       // outputs indexed by row0_out
};

// per group: C[M, N] = A_g^T B_g over the rows of the group (K = rows of the group)
struct WGemm {
  const int4* ginfo;        // per launch index (descending rows): {group, rows, first row, compact slot}; NULL: identity
  int32_t n_rows;
  int32_t M, N;
  const void* A;            // element (row, m) at A + row*lda + m
  int64_t lda;
  int32_t a_per_group;      // shared mode: A rows of group g start at g*n_rows
  const void* B[2];         // element (row, n) at B + row*ldb + n; B[1]: second product (dual GEMM, or blockIdx.z = 1)
  int64_t ldb;
  int32_t b_per_group;
  void* C[2];
  int64_t c_slot;           // elements per slot
  int32_t k_min, k_max;     // only groups with k_min <= rows <= k_max are processed by this launch
  int32_t n_reps;           // consecutive column tiles per block (0 or 1: one)
};

}  // namespace moe
