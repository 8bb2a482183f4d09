// Grouped GEMM of the expert computation: argument block and launcher, shared by the forward
// (ffn.hip) and backward (ffn_backward.hip) translation units.  Not part of the public ABI.
#pragma once
#include "common.h"

namespace occult {

struct GemmArgs {
  const void* A;            // activation rows, K-contiguous
  int lda;                  // elements between A rows
  const int32_t* a_rows;    // [rows] source row of each logical row, or NULL (identity)
  const void* B;            // weights [group][N][kseg]
  const void* B2;           // second weight matrix (up projection) when SWIGLU, same layout
  const void* Bp;           // the same weights in the weight-streaming kernel's own order (occult_pack_weights),
                            // or NULL; read instead of B / B2 when that kernel is chosen
  long long bp_group_stride;   // bytes between consecutive weight matrices (pairs, when SWIGLU) in Bp
  long long b_group_stride; // elements between consecutive weight matrices
  int ldb;                  // elements between B rows (= kseg)
  int kseg;                 // K elements held by one weight matrix; K > kseg walks consecutive matrices
  void* C;                  // output rows
  int ldc;                  // elements between C rows
  int c_col0;               // first output column written by group 0
  int c_group_cols;         // group g writes from column c_col0 + g * c_group_cols
  void* C2;                 // SWIGLU only, or NULL: the two pre-activations are stored as well, in rows of 2 * ldc
                            // elements: [gate | up] of group g from column 2 * (c_col0 + g * c_group_cols), the up
                            // half N columns after the gate half
  const int32_t* grp_offset;  // [ngroups+1] logical-row prefix per group, or NULL: every group takes rows [0, M)
  const int32_t* grp_widx;    // [ngroups] weight matrix of each group, or NULL: w_base + group
  int w_base;
  int ngroups;
  int M;                    // rows when grp_offset == NULL
  int a_rows_total;         // rows of the A buffer that may be addressed (bounds 32-bit offsets)
  int plain_map;            // small-tile kernel: workgroup id = m-tile * n_tiles + n-tile (tiny grids)
  int ksplit;               // small-tile kernel, one group, no SWIGLU: blockIdx.y takes K tiles
                            // [y*nk/ksplit, (y+1)*nk/ksplit) and writes f32 sums to ws; 0 or 1 = off
  float* ws;                // [ksplit][M][N] partial sums
  int N;                    // output columns (for SWIGLU: columns of h)
  int K;
};

// Launches C[rows][N] = A[rows][K] x B[group][N][K]^T group by group (cfg.dtype: bf16 on MFMA with f32
// accumulation, or plain f32); with `swiglu` the output is silu(A B^T) * (A B2^T).  `total_rows` = logical
// rows over all groups.  Picks the tile shape from the rows per group.  Returns an OCCULT_* code.
int launch_gemm(const occult_cfg_t& c, const GemmArgs& a, bool swiglu, int total_rows, hipStream_t s);

}  // namespace occult
