// Backward pass of the expert computation: weight gradients of the grouped SwiGLU experts.
//
// Same sources as ffn_backward.hip (the paper trains through the layer and prints no backward
// algorithm; this is the chain rule through the forward's expert on the same plan).  For the
// expert at placement position P with EPD rows q in [exp_offset[P], exp_offset[P+1]):
//   dW_down = sum_q epd_dy[q] (x) epd_h[q]          [d][f]
//   dW_gate = sum_q dg[q] (x) x_q,  dW_up = sum_q du[q] (x) x_q     [f][d],  x_q = sfd_x[epd_sfd_row[q]]
// i.e. per expert C[m][n] = sum over its rows r of A[r][m] * B[src(r)][n]: a contraction over the
// ROW index of two row-major operands, the one GEMM shape the forward kernels do not cover (their
// operands are both contiguous along the contracted index).
//
// bf16 kernel (namespace wgd below).  Block = 256 threads = 4 waves (2 x 2), block tile 256 x 256
// outputs, wave tile 128 x 128 = 4 x 4 v_mfma_f32_32x32x16_bf16 tiles (256 accumulator registers, one
// block per CU).  Outputs are f32 (gradient accumulation across calls is exact to f32), stored
// straight from the accumulators: 32 lanes cover 128 contiguous bytes.  With 8 groups or more a
// group's tiles are launched on one XCD (workgroup id % 8), so its rows are fetched into one L2.
#include "common.h"

namespace occult {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct WgradArgs {
  const void* A;             // [rows][lda]: its columns index the output rows (M of them)
  int lda, a_col0, a_group_cols;   // group g reads columns a_col0 + g * a_group_cols ...
  const void* B;             // [rows][ldb]: its columns index the output columns (N of them)
  int ldb, b_col0, b_group_cols;
  const int32_t* b_rows;     // [rows] source row in B of each logical row, or NULL (identity)
  float* C;                  // [matrix][M][ldc]
  long long c_mat_stride;
  int ldc;
  const int32_t* grp_offset; // [ngroups+1] logical-row range per group, or NULL: every group takes rows [0, R)
  const int32_t* grp_widx;   // [ngroups] output matrix of each group, or NULL: w_base + group
  int w_base, ngroups, R;
  int M, N;
  int accumulate;            // 0: C = product, 1: C += product
  int rsplit;                // uniform groups only (grp_offset == NULL): the R rows are cut into rsplit slices of
                             // rslice rows (a multiple of the step), each a workgroup of its own that writes its f32
                             // partial product to ws[slice][group][M][N]; wgrad_reduce adds the slices in order.
                             // 0 or 1: no split
  int rslice;
  float* ws;
};

// ------------------------------------------------------------------------------------------
// The MFMA operands want 8 consecutive contracted elements per lane, which in memory are 8
// different rows.  A first version staged the operands through registers (16-byte loads of 4 rows,
// a 4 x 8 transpose with v_perm_b32, 8-byte LDS writes): it can keep only one step of operands
// (64 KiB per CU) in flight, which covers a step's products but not the latency of memory under
// load (measured: products alone 985 TFLOP/s, with the loads 480).  Here a step is 32 rows, the raw
// row-major tiles go from global memory straight into a ring of NST LDS stages
// (global_load_lds_dwordx4: no registers held while a load is in flight), NST - 1 steps ahead, and
// the transposition happens in the fragment reads: ds_read_b64_tr_b16 gives every lane
// of a 16-lane block the 4 contracted elements of its own column out of 4 rows x 16 columns that the
// block's lanes address (lanes 4e..4e+3 address row e).  Two such reads make one MFMA operand.
// One load instruction fills 1 KiB = 2 tile rows; 16-byte chunk c of tile row k sits at chunk
// c ^ ((k & 3) << 2) (realised by the loading lane's choice of source chunk), so that the 4 rows x
// 64 bytes a block reads fall on different banks.  Rows past the group's end: the A side reads a
// page of zeros, the B side repeats the group's last row (0 * finite = 0).  Gathered row indices
// take the same road two steps ahead of the rows they address: one 4-byte-per-lane LDS-directed
// load per wave and step into a small ring, read back with ordinary LDS reads.  Every step issues
// the same number of loads (steps past the end are clamped like rows past the end), so one
// constant vmcnt tells that the current step's tiles, and the indices about to be used, have landed.
namespace wgd {
constexpr int BM = 256, BN = 256, BK = 32;
constexpr int NST = 4;   // the index ring below assumes 4
constexpr int OP_BYTES = BK * 512;          // raw operand tile: 32 rows x 256 columns of bf16
constexpr int STAGE_BYTES = 2 * OP_BYTES;   // 32 KiB

__device__ __attribute__((aligned(16))) const unsigned zero_page[4] = {0u, 0u, 0u, 0u};

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// 64 lanes x 16 bytes from per-lane global addresses to LDS [lds, lds + 1024); counted by vmcnt
__device__ __forceinline__ void load_to_lds_16(const char* src, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(src) : "memory", "m0");
}
// the same with a wave-uniform base and a 32-bit byte offset per lane
__device__ __forceinline__ void load_to_lds_16(const char* base, unsigned off, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(off), "s"(base)
               : "memory", "m0");
}
// 64 lanes x 4 bytes to LDS [lds, lds + 256)
__device__ __forceinline__ void load_to_lds_4(const char* src, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds), "v"(src) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}
#pragma clang diagnostic pop

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

template <bool GATHER>   // B rows through a.b_rows
__global__ __launch_bounds__(256) void wgrad_bf16(const WgradArgs a) {
  __shared__ __attribute__((aligned(1024))) char smem[NST * STAGE_BYTES];
  __shared__ __attribute__((aligned(256))) int s_idx[4][4][64];   // [wave][step % 4][row of the wave's 8, repeated]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int nt_n = (a.N + BN - 1) / BN;
  const int tiles = ((a.M + BM - 1) / BM) * nt_n;
  // with 8 groups or more a group's tiles share an XCD (and its L2); fewer groups (shared experts: few
  // groups of many rows) are spread over all XCDs instead
  int group, tile, slice = 0;
  if (a.ngroups >= 8) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    group = (slot / tiles) * 8 + xcd;
    tile = slot % tiles;
  } else {
    const int per_slice = a.ngroups * tiles;
    const int bid = blockIdx.x % per_slice;
    slice = __builtin_amdgcn_readfirstlane(blockIdx.x / per_slice);   // 0 unless the rows are split (host: grid = slices * per_slice)
    group = bid / tiles;
    tile = bid % tiles;
  }
  if (group >= a.ngroups) return;   // whole block; before any barrier
  const bool split = a.rsplit > 1;
  // (the division runs in vector registers; the tile origin feeds scalar operands of the loads below)
  const int m0 = __builtin_amdgcn_readfirstlane((tile / nt_n) * BM), n0 = __builtin_amdgcn_readfirstlane((tile % nt_n) * BN);
  int r0 = 0, r1 = a.R;
  if (a.grp_offset) {
    r0 = a.grp_offset[group];
    r1 = a.grp_offset[group + 1];
  } else if (split) {
    r0 = min(a.R, slice * a.rslice);
    r1 = min(a.R, r0 + a.rslice);
  }
  r0 = __builtin_amdgcn_readfirstlane(r0);
  r1 = __builtin_amdgcn_readfirstlane(r1);
  const long long widx = a.grp_widx ? a.grp_widx[group] : (a.w_base + group);
  const int nk = (r1 - r0 + BK - 1) / BK;

  f32x16 acc[4][4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.0f;

  if (nk > 0) {
    // loader role: a load instruction covers tile rows kb, kb + 1; lane = (row rr, chunk position p)
    const int rr = lane >> 5, p = lane & 31;
    const char* a_cols = static_cast<const char*>(a.A) + (long long)(a.a_col0 + group * a.a_group_cols + m0) * 2;
    const char* b_cols = static_cast<const char*>(a.B) + (long long)(a.b_col0 + group * a.b_group_cols + n0) * 2;
    const long long a_pitch = (long long)a.lda * 2, b_pitch = (long long)a.ldb * 2;
    const int a_chunks = min(32, (a.M - m0) / 8), b_chunks = min(32, (a.N - n0) / 8);   // valid 16-byte chunks per row
    const unsigned smem_base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;   // LDS byte address
    const char* zeros = reinterpret_cast<const char*>(zero_page);

    // per-lane byte offsets of the 4 loads per operand inside a step's 32 rows: constant over the steps
    unsigned off_a[4], off_b[4], chunk_b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = wave * 8 + i * 2 + rr;           // tile row of this lane
      int ca = p ^ ((k & 3) << 2), cb = ca;          // source chunk of this lane's position
      if (ca >= a_chunks) ca = 0;                     // columns past M or N: any valid chunk (never stored)
      if (cb >= b_chunks) cb = 0;
      off_a[i] = (unsigned)(k * a_pitch + ca * 16);
      off_b[i] = (unsigned)(k * b_pitch + cb * 16);
      chunk_b[i] = (unsigned)(cb * 16);
    }
    // the same for a step holding the group's last rows, or past them (issued to keep the load count constant)
    auto issue_tail = [&](int s) {
      const unsigned st = smem_base + (unsigned)(s % NST) * STAGE_BYTES;
      const int row0 = r0 + s * BK;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kb = wave * 8 + i * 2;               // tile rows kb, kb + 1
        const long long ra = row0 + kb + rr;
        // A: rows past the end read zeros
        const char* src_a = (ra < r1) ? a_cols + ra * a_pitch + (off_a[i] - (unsigned)((kb + rr) * a_pitch)) : zeros;
        load_to_lds_16(src_a, st + (unsigned)kb * 512u);
        // B: rows past the end repeat the last row (the fetched indices are clamped the same way)
        long long rb = min(row0 + kb + rr, r1 - 1);
        if (GATHER) rb = s_idx[wave][s & 3][i * 2 + rr];
        load_to_lds_16(b_cols + rb * b_pitch + chunk_b[i], st + (unsigned)OP_BYTES + (unsigned)kb * 512u);
      }
    };
    auto issue = [&](int s) {   // the 8 loads of this wave for step s into stage s % NST
      const unsigned st = smem_base + (unsigned)(s % NST) * STAGE_BYTES;
      const int row0 = r0 + s * BK;                    // first row of the step
      if (row0 + BK <= r1) {   // block-uniform: every row inside the group, addresses = uniform base + constant offsets
        const char* a_step = a_cols + (long long)row0 * a_pitch;
        const char* b_step = b_cols + (long long)row0 * b_pitch;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned kb = (unsigned)(wave * 8 + i * 2);
          load_to_lds_16(a_step, off_a[i], st + kb * 512u);
          if (GATHER) {
            const long long rb = s_idx[wave][s & 3][i * 2 + rr];   // fetched two steps ago
            load_to_lds_16(b_cols + rb * b_pitch + chunk_b[i], st + (unsigned)OP_BYTES + kb * 512u);
          } else {
            load_to_lds_16(b_step, off_b[i], st + (unsigned)OP_BYTES + kb * 512u);
          }
        }
      } else {
        issue_tail(s);
      }
    };

    // fragment reads: lane l = 16 b + j, j = 4 e + q: block b covers columns 16 (b & 1) .. + 16 and rows
    // 8 (b >> 1) + e (first read), + 4 (second read); the lane addresses 4 columns (8 bytes) of row e
    const int fb = lane >> 4, fe = (lane >> 2) & 3, fq = lane & 3;
    const int f_row = 8 * (fb >> 1) + fe;                       // + 16 * ks, + 4 for the second read
    const int f_col4 = 4 * (fb & 1) + fq;                       // 8-byte unit inside the 32-column block
    typedef __attribute__((address_space(3))) char lds_char;
    auto frag = [&](const lds_char* op, int col0, int ks) -> bf16x8 {   // col0: first column of the 32-column block
      const int row = ks * 16 + f_row;
      const int unit = (col0 >> 2) + f_col4;                    // 8-byte unit inside the tile row
      const int pos = ((unit >> 1) ^ (fe << 2)) * 16 + (unit & 1) * 8;
      const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
          (bf16x4 __attribute__((address_space(3)))*)(op + row * 512 + pos));
      const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
          (bf16x4 __attribute__((address_space(3)))*)(op + (row + 4) * 512 + pos));
      return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto read_frags = [&](int s, int ks, bf16x8 (&fa)[4], bf16x8 (&fbv)[4]) {
      const lds_char* As = (const lds_char*)smem + (s % NST) * STAGE_BYTES;
      const lds_char* Bs = As + OP_BYTES;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        fa[i] = frag(As, wm * 128 + i * 32, ks);
        fbv[i] = frag(Bs, wn * 128 + i * 32, ks);
      }
    };
    auto mma = [&](const bf16x8 (&fa)[4], const bf16x8 (&fbv)[4]) {
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fbv[ni], acc[mi][ni], 0, 0, 0);
    };

    // source rows of this wave's 8 tile rows of step s (clamped to the group) -> its ring slot s % 4
    const unsigned idx_base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)&s_idx[wave][0][0];
    auto issue_idx = [&](int s) {
      const int r = min(r0 + s * BK + wave * 8 + (lane & 7), r1 - 1);
      load_to_lds_4(reinterpret_cast<const char*>(a.b_rows + r), idx_base + (unsigned)(s & 3) * 256u);
    };
    constexpr int OPS = GATHER ? 9 : 8;   // loads per wave and step
    if (GATHER) {
#pragma unroll
      for (int s = 0; s < 4; ++s) issue_idx(s);          // one ring of indices
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // a wave reads only its own indices: no barrier
    }
    // The prologue issues in the order the loop continues: indices of step NST go into the slot step 0 has just
    // been read from (its reads have returned: the tile loads' addresses depend on them), BEFORE the tiles of
    // steps 1 and 2, so that the constant count below covers them when step 1 reads them.
    issue(0);
    if (GATHER) issue_idx(NST);
#pragma unroll
    for (int s = 1; s < NST - 1; ++s) issue(s);
    // Loads complete in order.  Per step a wave issues [indices of step s + NST + 1,] 8 tile loads of step
    // s + NST - 1.  The tiles of step s are older than the (NST - 2) * OPS loads of the last NST - 2 steps;
    // the indices used (step s + NST - 1, issued first two steps ago) are older than all but one of them.
    // After the barrier every wave's tiles of step s are in LDS, and every wave is done with the stage that
    // step s + NST - 1 overwrites.
    // Two loops, so that neither has a branch inside (one would make the register allocator move the 256
    // accumulators around): first the steps whose prefetched step lies wholly inside the group.
    const int n_main = max(0, (r1 - r0) / BK - (NST - 1));
    int s = 0;
    for (; s < n_main; ++s) {
      wait_loads_and_barrier<(NST - 2) * OPS - (GATHER ? 1 : 0)>();
      bf16x8 fa[2][4], fbv[2][4];
      read_frags(s, 0, fa[0], fbv[0]);
      __builtin_amdgcn_sched_barrier(0);
      const int sn = s + NST - 1;
      if (GATHER) issue_idx(s + NST + 1);
      // With one wave per SIMD nothing hides an instruction clump: the first half's 16 products are issued as
      // 8 groups of {2 MFMAs, 1 tile load, 1 fragment read for the second half}, pinned in source order.
      const unsigned st = smem_base + (unsigned)(sn % NST) * STAGE_BYTES;
      const char* a_step = a_cols + (long long)(r0 + sn * BK) * a_pitch;
      const char* b_step = b_cols + (long long)(r0 + sn * BK) * b_pitch;
      const lds_char* As = (const lds_char*)smem + (s % NST) * STAGE_BYTES;
      const lds_char* Bs = As + OP_BYTES;
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        const int mi = g >> 1, nj = (g & 1) * 2;
        acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][mi], fbv[0][nj], acc[mi][nj], 0, 0, 0);
        acc[mi][nj + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][mi], fbv[0][nj + 1], acc[mi][nj + 1], 0, 0, 0);
        const int i = g & 3;
        const unsigned kb = (unsigned)(wave * 8 + i * 2);
        if (g < 4) {
          load_to_lds_16(a_step, off_a[i], st + kb * 512u);
          fa[1][g] = frag(As, wm * 128 + g * 32, 1);
        } else {
          if (GATHER) {
            const long long rb = s_idx[wave][sn & 3][i * 2 + rr];   // fetched two steps ago
            load_to_lds_16(b_cols + rb * b_pitch + chunk_b[i], st + (unsigned)OP_BYTES + kb * 512u);
          } else {
            load_to_lds_16(b_step, off_b[i], st + (unsigned)OP_BYTES + kb * 512u);
          }
          fbv[1][g - 4] = frag(Bs, wn * 128 + (g - 4) * 32, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      mma(fa[1], fbv[1]);
    }
    // then the steps that prefetch the group's last rows or past them
    for (; s < nk; ++s) {
      wait_loads_and_barrier<(NST - 2) * OPS - (GATHER ? 1 : 0)>();
      bf16x8 fa[2][4], fbv[2][4];
      read_frags(s, 0, fa[0], fbv[0]);
      if (GATHER) issue_idx(s + NST + 1);
      issue_tail(s + NST - 1);
      read_frags(s, 1, fa[1], fbv[1]);
      mma(fa[0], fbv[0]);
      mma(fa[1], fbv[1]);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the clamped loads past the end, before the block's LDS is released
  }

  // accumulator element e of lane l: output row (e / 4) * 8 + (l / 32) * 4 + e % 4, column l % 32 of its 32 x 32 tile.
  // Stores (and, when accumulating, loads) go through a buffer descriptor over the wave tile's valid rows: rows
  // past M lie beyond its range and are dropped by the hardware, columns past N are sent there: no branches.
  const int frow = lane & 31, fk = lane >> 5;
  const int rows_left = min(a.M - (m0 + wm * 128), 128);
  const int cols_left = min(a.N - (n0 + wn * 128), 128);
  // a row slice writes its partial product densely into the scratch tensor [slice][group][M][N] instead
  const int ldc = split ? a.N : a.ldc;
  const bool accumulate = !split && a.accumulate;
  float* c_mat = split ? a.ws + ((long long)slice * a.ngroups + group) * ((long long)a.M * a.N) : a.C + widx * a.c_mat_stride;
  const unsigned n_rec = rows_left > 0 && cols_left > 0 ? (unsigned)((rows_left - 1) * ldc + cols_left) * 4u : 0u;
  const unsigned long long c_tile = reinterpret_cast<unsigned long long>(
      c_mat + (long long)(m0 + wm * 128) * ldc + n0 + wn * 128);
  const unsigned long long c_tile_u =   // the descriptor has to sit in scalar registers
      ((unsigned long long)__builtin_amdgcn_readfirstlane((unsigned)(c_tile >> 32)) << 32) |
      (unsigned)__builtin_amdgcn_readfirstlane((unsigned)c_tile);
  const __amdgpu_buffer_rsrc_t c_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      reinterpret_cast<void*>(c_tile_u), 0, __builtin_amdgcn_readfirstlane((int)n_rec), 0x00020000);
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int nl = ni * 32 + frow;
      unsigned off[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int ml = mi * 32 + (e >> 2) * 8 + fk * 4 + (e & 3);
        off[e] = nl < cols_left ? (unsigned)(ml * ldc + nl) * 4u : n_rec;
      }
      if (accumulate) {   // block-uniform; the 16 loads of a tile are in flight together
        float old[16];
#pragma unroll
        for (int e = 0; e < 16; ++e)
          old[e] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(c_rsrc, (int)off[e], 0, 0));
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mi][ni][e] += old[e];
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float v = acc[mi][ni][e];   // (a bit cast applied to the vector element itself stores element 0 sixteen times)
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), c_rsrc, (int)off[e], 0, 0);
      }
    }
}
}  // namespace wgd

// Adds the row slices' partial products in slice order and writes (or adds) the sum: C[group] (=|+=) ws[0][group]
// + ws[1][group] + ...  One thread per 4 output columns (host: N % 4 == 0, ldc % 4 == 0, 16-byte aligned bases).
__global__ __launch_bounds__(256) void wgrad_reduce(const WgradArgs a) {
  const long long quads_per_mat = (long long)a.M * (a.N / 4);
  const long long total = quads_per_mat * a.ngroups;
  const long long slice_stride = (long long)a.ngroups * a.M * a.N;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int group = (int)(i / quads_per_mat);
    const long long q = i - group * quads_per_mat;
    const int m = (int)(q / (a.N / 4)), n = (int)(q - (long long)m * (a.N / 4)) * 4;
    const float* src = a.ws + (long long)group * a.M * a.N + (long long)m * a.N + n;
    f32x4 sum = *reinterpret_cast<const f32x4*>(src);
    for (int sl = 1; sl < a.rsplit; ++sl) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(src + sl * slice_stride);
      sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    const long long widx = a.grp_widx ? a.grp_widx[group] : (a.w_base + group);
    f32x4* dst = reinterpret_cast<f32x4*>(a.C + widx * a.c_mat_stride + (long long)m * a.ldc + n);
    if (a.accumulate) {
      const f32x4 old = *dst;
      sum.x += old.x; sum.y += old.y; sum.z += old.z; sum.w += old.w;
    }
    *dst = sum;
  }
}

// f32 path for parity-sized layers: one thread per output element, rows summed in order
__global__ __launch_bounds__(256) void wgrad_f32(const WgradArgs a) {
  const int group = blockIdx.z;
  const int m = blockIdx.y * 16 + (threadIdx.x >> 4), n = blockIdx.x * 16 + (threadIdx.x & 15);
  if (m >= a.M || n >= a.N) return;
  int r0 = 0, r1 = a.R;
  if (a.grp_offset) {
    r0 = a.grp_offset[group];
    r1 = a.grp_offset[group + 1];
  }
  const long long widx = a.grp_widx ? a.grp_widx[group] : (a.w_base + group);
  const float* A = static_cast<const float*>(a.A) + a.a_col0 + group * a.a_group_cols + m;
  const float* B = static_cast<const float*>(a.B) + a.b_col0 + group * a.b_group_cols + n;
  float sum = 0.0f;
  for (int r = r0; r < r1; ++r) {
    const long long src = a.b_rows ? a.b_rows[r] : r;
    sum = fmaf(A[(long long)r * a.lda], B[src * a.ldb], sum);
  }
  float* p = a.C + widx * a.c_mat_stride + (long long)m * a.ldc + n;
  *p = a.accumulate ? *p + sum : sum;
}

// Row slices for a product with fewer than 8 uniform groups of many rows (shared experts of a large batch): its
// groups x tiles workgroups alone leave most of the chip idle.  Returns the number of slices (1 = no split) that
// minimises rounds of workgroups x rows per slice, at most 8, each of at least 2048 rows; *rslice = rows per slice.
static int choose_row_split(const occult_cfg_t& c, int ngroups, int M, int N, int R, int* rslice) {
  *rslice = R;
  if (c.dtype != OCCULT_BF16 || ngroups <= 0 || ngroups >= 8 || N % 4 != 0) return 1;
  static int cached_cus = 0;   // compute units of the device first asked about (one kind of GPU per process)
  if (cached_cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cached_cus = n;
    else
      cached_cus = 256;
  }
  const int cus = cached_cus;
  const long long tiles = (long long)((M + wgd::BM - 1) / wgd::BM) * ((N + wgd::BN - 1) / wgd::BN) * ngroups;
  int best = 1;
  double best_cost = (double)((tiles + cus - 1) / cus) * R;
  for (int r = 2; r <= 8; ++r) {
    const int rows = ((R + r - 1) / r + wgd::BK - 1) / wgd::BK * wgd::BK;
    if (rows < 2048) break;
    const double cost = (double)((tiles * r + cus - 1) / cus) * rows;
    if (cost < best_cost * 0.95) {
      best = r;
      best_cost = cost;
      *rslice = rows;
    }
  }
  return best;
}

static int launch_wgrad(const occult_cfg_t& c, const WgradArgs& a, hipStream_t s) {
  if (a.ngroups == 0 || a.M == 0 || a.N == 0) return OCCULT_OK;
  if (c.dtype == OCCULT_BF16) {
    const long long tiles = (long long)((a.M + wgd::BM - 1) / wgd::BM) * ((a.N + wgd::BN - 1) / wgd::BN);
    long long blocks = a.ngroups >= 8 ? (long long)((a.ngroups + 7) / 8) * tiles * 8 : (long long)a.ngroups * tiles;
    if (a.rsplit > 1) blocks *= a.rsplit;
    OCC_REQUIRE(blocks < (1ll << 31), OCCULT_EINVAL, "weight-gradient grid too large");
    if (a.b_rows) hipLaunchKernelGGL(wgd::wgrad_bf16<true>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(wgd::wgrad_bf16<false>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    if (a.rsplit > 1) {
      OCC_LAUNCH_CHECK("wgrad");
      hipLaunchKernelGGL(wgrad_reduce, dim3(2048), dim3(256), 0, s, a);
    }
  } else {
    OCC_REQUIRE(a.ngroups <= 65535, OCCULT_EINVAL, "too many groups");
    hipLaunchKernelGGL(wgrad_f32, dim3((a.N + 15) / 16, (a.M + 15) / 16, a.ngroups), dim3(256), 0, s, a);
  }
  OCC_LAUNCH_CHECK("wgrad");
  return OCCULT_OK;
}

}  // namespace occult

using namespace occult;

// chooses the row split of a uniform-group product when the caller's scratch holds its partial sums
static void set_row_split(const occult_cfg_t& c, WgradArgs& a, void* ws, size_t ws_bytes) {
  a.rsplit = 0;
  if (!ws) return;
  int rslice = 0;
  const int r = choose_row_split(c, a.ngroups, a.M, a.N, a.R, &rslice);
  if (r > 1 && ws_bytes >= (size_t)r * a.ngroups * a.M * a.N * sizeof(float)) {
    a.rsplit = r;
    a.rslice = rslice;
    a.ws = static_cast<float*>(ws);
  }
}

// scratch for the row-split products of the shared experts: the largest of the three (they run one after another)
static size_t wgrad_ws_need(const occult_cfg_t& c) {
  if (c.S <= 0 || c.T <= 0) return 0;
  int rs = 0;
  const int r1 = choose_row_split(c, c.S, c.d, c.f, c.T, &rs);
  const int r2 = choose_row_split(c, c.S, c.f, c.d, c.T, &rs);
  const int r = r1 > r2 ? r1 : r2;
  return r > 1 ? (size_t)r * c.S * c.d * c.f * sizeof(float) : 0;
}

extern "C" int occult_expert_ffn_backward_weights_ws_bytes(const occult_cfg_t* cfg, size_t* ws_bytes) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  OCC_REQUIRE(ws_bytes, OCCULT_ENULLPTR, "ws_bytes is NULL");
  *ws_bytes = wgrad_ws_need(*cfg);
  return OCCULT_OK;
}

static int backward_weights_impl(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                 const void* x, const void* epd_h, const void* h_shared,
                                 const void* epd_dy, const void* dy, const void* epd_gu,
                                 const void* gu_shared, float* dw_gate, float* dw_up, float* dw_down,
                                 int accumulate, void* ws, size_t ws_bytes, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  OCC_REQUIRE(aligned16(ws), OCCULT_EALIGN, "ws is not 16-byte aligned");
  OCC_REQUIRE(dw_gate && dw_up && dw_down, OCCULT_ENULLPTR, "dw_gate, dw_up or dw_down is NULL");
  OCC_REQUIRE(accumulate == 0 || accumulate == 1, OCCULT_EINVAL, "accumulate=%d must be 0 or 1", accumulate);
  const int es = elem_size(c);
  OCC_REQUIRE(((size_t)c.d * es) % 16 == 0 && ((size_t)c.f * es) % 16 == 0, OCCULT_EALIGN,
              "rows of d=%d or f=%d elements are not multiples of 16 bytes", c.d, c.f);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const long long mat = (long long)c.f * c.d;
  OCC_REQUIRE(plan && plan->exp_offset && plan->pos_expert && plan->epd_sfd_row, OCCULT_ENULLPTR,
              "plan or one of its tables is NULL");
  if (c.T > 0) {   // with no rows nothing is read and the products below write zeros (or add nothing)
    OCC_REQUIRE(sfd_x && epd_h && epd_dy && epd_gu, OCCULT_ENULLPTR, "sfd_x, epd_h, epd_dy or epd_gu is NULL");
    if (c.S > 0)
      OCC_REQUIRE(x && h_shared && dy && gu_shared, OCCULT_ENULLPTR, "x, h_shared, dy or gu_shared is NULL with S=%d",
                  c.S);
  }
  OCC_REQUIRE(aligned16(sfd_x) && aligned16(x) && aligned16(epd_h) && aligned16(h_shared) && aligned16(epd_dy) &&
                  aligned16(dy) && aligned16(epd_gu) && aligned16(gu_shared),
              OCCULT_EALIGN, "a buffer is not 16-byte aligned");

  WgradArgs routed{};
  routed.grp_offset = plan->exp_offset; routed.grp_widx = plan->pos_expert; routed.ngroups = c.E;
  routed.accumulate = accumulate;
  WgradArgs shared{};
  shared.grp_offset = nullptr; shared.grp_widx = nullptr; shared.w_base = c.E; shared.ngroups = c.S; shared.R = c.T;
  shared.accumulate = accumulate;
  for (int part = 0; part < (c.S > 0 ? 2 : 1); ++part) {
    const bool sh = part == 1;
    const WgradArgs& base = sh ? shared : routed;
    {   // dW_down [d][f] = sum_r dy_r (x) h_r
      WgradArgs a = base;
      a.A = sh ? dy : epd_dy; a.lda = c.d; a.M = c.d;
      a.B = sh ? h_shared : epd_h; a.ldb = sh ? c.S * c.f : c.f; a.b_group_cols = sh ? c.f : 0; a.N = c.f;
      a.C = dw_down; a.c_mat_stride = mat; a.ldc = c.f;
      if (sh) set_row_split(c, a, ws, ws_bytes);
      rc = launch_wgrad(c, a, s);
      if (rc) return rc;
    }
    for (int up = 0; up < 2; ++up) {   // dW_gate, dW_up [f][d] = sum_r dg_r (x) x_r, sum_r du_r (x) x_r
      WgradArgs a = base;
      a.A = sh ? gu_shared : epd_gu; a.lda = sh ? c.S * 2 * c.f : 2 * c.f; a.a_col0 = up ? c.f : 0;
      a.a_group_cols = sh ? 2 * c.f : 0; a.M = c.f;
      a.B = sh ? x : sfd_x; a.ldb = c.d; a.b_rows = sh ? nullptr : plan->epd_sfd_row; a.N = c.d;
      a.C = up ? dw_up : dw_gate; a.c_mat_stride = mat; a.ldc = c.d;
      if (sh) set_row_split(c, a, ws, ws_bytes);
      rc = launch_wgrad(c, a, s);
      if (rc) return rc;
    }
  }
  return OCCULT_OK;
}

extern "C" int occult_expert_ffn_backward_weights(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                                  const void* x, const void* epd_h, const void* h_shared,
                                                  const void* epd_dy, const void* dy, const void* epd_gu,
                                                  const void* gu_shared, float* dw_gate, float* dw_up, float* dw_down,
                                                  int accumulate, occult_stream_t stream) {
  return backward_weights_impl(cfg, plan, sfd_x, x, epd_h, h_shared, epd_dy, dy, epd_gu, gu_shared, dw_gate, dw_up, dw_down,
                               accumulate, nullptr, 0, stream);
}

extern "C" int occult_expert_ffn_backward_weights_ws(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                                     const void* x, const void* epd_h, const void* h_shared,
                                                     const void* epd_dy, const void* dy, const void* epd_gu,
                                                     const void* gu_shared, float* dw_gate, float* dw_up, float* dw_down,
                                                     int accumulate, void* ws, size_t ws_bytes, occult_stream_t stream) {
  return backward_weights_impl(cfg, plan, sfd_x, x, epd_h, h_shared, epd_dy, dy, epd_gu, gu_shared, dw_gate, dw_up, dw_down,
                               accumulate, ws, ws_bytes, stream);
}
