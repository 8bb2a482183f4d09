// occult_expert_ffn: grouped SwiGLU expert computation (paper App. A.2 "SMM with Scattering" and
// the matrix product of "SMM with Merging"; Sec. 3.1: each operator bridges two tensor states).
//
//   GEMM-1 (SFD -> EPD): for the expert at placement position P, its EPD rows
//     [exp_offset[P], exp_offset[P+1]) gather their A rows from sfd_x through epd_sfd_row (the
//     replication happens in the load, no expanded copy of the input exists); B = [W_gate; W_up];
//     the epilogue applies silu(gate) * up and stores bf16 epd_h.
//   GEMM-2 (EPD -> EPD): epd_y rows = epd_h rows x W_down^T.  The reduction over a device's
//     experts is left to combine's first stage (order-fixed, no float atomics).
//   Shared experts: the same two kernels over all T rows of x with the shared weights.
//
// bf16 path: LDS-tiled MFMA (v_mfma_f32_32x32x16_bf16), f32 accumulation.  Weights are
// K-contiguous ([out][in]), activations are K-contiguous rows, so both MFMA operands are read
// from LDS as 16-byte K-runs and no transpose is needed.
// f32 path: plain f32 FMA kernel for small parity-sized layers.
#include "common.h"

namespace occult {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GemmArgs {
  const void* A;            // activation rows, K-contiguous
  int lda;                  // elements between A rows
  const int32_t* a_rows;    // [rows] source row of each logical row, or NULL (identity)
  const void* B;            // weights [group][N][kseg]
  const void* B2;           // second weight matrix (up projection) when SWIGLU, same layout
  long long b_group_stride; // elements between consecutive weight matrices
  int ldb;                  // elements between B rows (= kseg)
  int kseg;                 // K elements held by one weight matrix; K > kseg walks consecutive matrices
  void* C;                  // output rows
  int ldc;                  // elements between C rows
  int c_col0;               // first output column written
  const int32_t* grp_offset;  // [ngroups+1] logical-row prefix per group, or NULL: one group of M rows
  const int32_t* grp_widx;    // [ngroups] weight matrix of each group, or NULL: w_base + group
  int w_base;
  int ngroups;
  int M;                    // rows when grp_offset == NULL
  int a_rows_total;         // rows of the A buffer that may be addressed (bounds 32-bit offsets)
  int N;                    // output columns (for SWIGLU: columns of h)
  int K;
};

struct TileInfo {
  int group, m0, rows, row_base;
};

// Workgroup id -> (m-tile, n-tile).  Workgroups are handed to the 8 XCDs round-robin and each XCD
// has its own L2, so the tiles an XCD runs at the same time should share operands: XCD x gets
// "chunks" x, x+8, ... of MC consecutive m-tiles times all n-tiles (about one tile per CU of the
// XCD), so that an A tile is fetched into one L2 only and a B tile is reused MC times there.
struct TileMap {
  int mt, nt;
};
__device__ __forceinline__ TileMap map_tile(int n_tiles) {
  const int mc = max(1, (32 + n_tiles / 2) / n_tiles);
  const int per_chunk = mc * n_tiles;
  const int b = blockIdx.x;
  const int xcd = b & 7, slot = b >> 3;
  const int chunk = (slot / per_chunk) * 8 + xcd;
  const int within = slot % per_chunk;
  TileMap tm;
  tm.mt = chunk * mc + within / n_tiles;
  tm.nt = within % n_tiles;
  return tm;
}
// grid size covering m_tiles x n_tiles under map_tile (host)
static long long mapped_grid(long long m_tiles, int n_tiles) {
  const int mc = (32 + n_tiles / 2) / n_tiles > 1 ? (32 + n_tiles / 2) / n_tiles : 1;
  long long chunks = (m_tiles + mc - 1) / mc;
  chunks = (chunks + 7) / 8 * 8;
  return chunks * mc * n_tiles;
}

// Which group and row block does m-tile `mt` fall in?  Group g owns ceil(rows_g / BM) tiles.
// Executed by every thread of the first wave; result through LDS.  group = -1: past the end.
template <int BM>
__device__ __forceinline__ TileInfo find_tile(const GemmArgs& a, int mt, TileInfo* s_info) {
  const int lane = threadIdx.x & 63;
  if (threadIdx.x < 64) {
    TileInfo ti;
    ti.group = -1;
    ti.m0 = ti.rows = ti.row_base = 0;
    if (a.grp_offset == nullptr) {
      if (mt * BM < a.M) {
        ti.group = 0;
        ti.m0 = mt * BM;
        ti.rows = a.M;
      }
      if (lane == 0) *s_info = ti;
    } else {
      if (lane == 0) *s_info = ti;
      int tiles_before = 0;
      for (int c0 = 0; c0 < a.ngroups; c0 += 64) {
        const int g = c0 + lane;
        const int lo = (g < a.ngroups) ? a.grp_offset[g] : 0;
        const int hi = (g < a.ngroups) ? a.grp_offset[g + 1] : 0;
        const int nt = (hi - lo + BM - 1) / BM;
        int incl = nt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int v = __shfl_up(incl, o, 64);
          if (lane >= o) incl += v;
        }
        const int excl = tiles_before + incl - nt;
        if (mt >= excl && mt < excl + nt) {   // at most one lane over all chunks
          ti.group = g;
          ti.m0 = (mt - excl) * BM;
          ti.rows = hi - lo;
          ti.row_base = lo;
          *s_info = ti;
        }
        tiles_before += __shfl(incl, 63, 64);
        if (tiles_before > mt) break;   // wave-uniform
      }
    }
  }
  __syncthreads();
  return *s_info;
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel, small tile (few rows per expert: decode-shaped layers).  Block = 256 threads = 4 waves (2 x 2), block tile 128 x 128 x 64,
// wave tile 64 x 64 = 2 x 2 MFMA tiles of 32 x 32.  With SWIGLU the 128 B-rows of a tile are
// [gate n0..n0+31 | up n0..n0+31 | gate n0+32..n0+63 | up n0+32..n0+63], so the two MFMA
// columns of a wave hold gate and up of the same 32 output columns.
namespace small {
constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_STRIDE = BK + 8;   // 144-byte rows: 16-byte reads of 8 consecutive rows hit 8 distinct bank groups

template <bool SWIGLU>
__global__ __launch_bounds__(256) void grouped_gemm_bf16(const GemmArgs a) {
  __shared__ __attribute__((aligned(16))) __bf16 As[BM * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) __bf16 Bs[BN * LDS_STRIDE];
  __shared__ TileInfo s_info;

  constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
  const int n_tiles = (a.N + BN_OUT - 1) / BN_OUT;
  const TileMap tm = map_tile(n_tiles);
  const int mt = tm.mt;
  const int n0 = tm.nt * BN_OUT;
  const TileInfo ti = find_tile<BM>(a, mt, &s_info);
  if (ti.group < 0) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const __bf16* A = static_cast<const __bf16*>(a.A);
  const long long widx = a.grp_widx ? a.grp_widx[ti.group] : (a.w_base + ti.group);

  // global -> LDS staging: thread owns 16-byte vector kv of rows (tid/8) + 32*i, i = 0..3
  const int kv = tid & 7, r_in = tid >> 3;
  const __bf16* a_src[4];
  const __bf16* b_src[4];   // row start inside the first weight matrix
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = r_in + 32 * i;
    int lr = ti.m0 + r;
    if (lr >= ti.rows) lr = ti.rows - 1;   // clamp: rows past the group are computed and dropped
    const int logical = ti.row_base + lr;
    const long long src = a.a_rows ? a.a_rows[logical] : logical;
    a_src[i] = A + src * a.lda + kv * 8;
    int ncol;
    const __bf16* wbase;
    if (SWIGLU) {
      const int blk = r >> 5, within = r & 31;
      ncol = n0 + (blk >> 1) * 32 + within;
      wbase = static_cast<const __bf16*>((blk & 1) ? a.B2 : a.B);
    } else {
      ncol = n0 + r;
      wbase = static_cast<const __bf16*>(a.B);
    }
    if (ncol >= a.N) ncol = a.N - 1;
    b_src[i] = wbase + widx * a.b_group_stride + (long long)ncol * a.ldb + kv * 8;
  }

  f32x16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.0f;

  const int nk = a.K / BK;
  u32x4 ga[4], gb[4];
  auto load_global = [&](int kt) {
    const int k0 = kt * BK;
    const int seg = k0 / a.kseg;                 // which weight matrix along K (shared down-proj)
    const long long boff = (long long)seg * a.b_group_stride + (k0 - seg * a.kseg);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ga[i] = *reinterpret_cast<const u32x4*>(a_src[i] + k0);
      gb[i] = *reinterpret_cast<const u32x4*>(b_src[i] + boff);
    }
  };
  load_global(0);

  for (int kt = 0; kt < nk; ++kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = r_in + 32 * i;
      *reinterpret_cast<u32x4*>(&As[r * LDS_STRIDE + kv * 8]) = ga[i];
      *reinterpret_cast<u32x4*>(&Bs[r * LDS_STRIDE + kv * 8]) = gb[i];
    }
    __syncthreads();
    if (kt + 1 < nk) load_global(kt + 1);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[2], fb[2];
      const int kof = kk * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
        fa[mi] = *reinterpret_cast<const bf16x8*>(&As[(wm * 64 + mi * 32 + (lane & 31)) * LDS_STRIDE + kof]);
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
        fb[ni] = *reinterpret_cast<const bf16x8*>(&Bs[(wn * 64 + ni * 32 + (lane & 31)) * LDS_STRIDE + kof]);
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
    }
    __syncthreads();
  }

  // epilogue.  Accumulator element r of lane l sits at row (r/4)*8 + (l/32)*4 + r%4, column l%32.
  __bf16* C = static_cast<__bf16*>(a.C);
  const int col_in = lane & 31;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = ti.m0 + wm * 64 + mi * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
      if (row >= ti.rows) continue;
      __bf16* crow = C + (long long)(ti.row_base + row) * a.ldc + a.c_col0;
      if (SWIGLU) {
        const int col = n0 + wn * 32 + col_in;
        if (col < a.N) {
          const float g = acc[mi][0][r], u = acc[mi][1][r];
          crow[col] = static_cast<__bf16>(g / (1.0f + __expf(-g)) * u);
        }
      } else {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          const int col = n0 + wn * 64 + ni * 32 + col_in;
          if (col < a.N) crow[col] = static_cast<__bf16>(acc[mi][ni][r]);
        }
      }
    }
  }
}
}  // namespace small

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel, main variant (prefill-shaped layers).  Block = 256 threads = 4 waves (2 x 2),
// block tile 256 x 256 x 64, wave tile 128 x 128 = 4 x 4 MFMA tiles of 32 x 32 (256 accumulator
// registers per lane, one wave per SIMD).
//
// Global -> LDS.  Operand tiles go from global memory straight into LDS
// (global_load_lds_dwordx4: no VGPR staging, no ds_write), double buffered: while tile kt is
// multiplied, tile kt+1 lands in the other stage.  The loads are issued from inline assembly
// (wave-uniform base in SGPRs + a 32-bit per-lane offset that is constant over K, so advancing K
// costs two scalar adds) and waited for with an explicit vmcnt: the compiler's own wait insertion
// treats an LDS-directed load as a FLAT access and could only wait for all outstanding loads at
// every LDS read.  One such load writes 64 lanes x 16 bytes contiguously = 8 rows of 128 bytes,
// so rows cannot be padded; bank conflicts of the 16-byte fragment reads are avoided by an XOR
// swizzle instead: chunk c of row r lives at slot c ^ ((r >> 1) & 7), realised by the loading
// lane's choice of global chunk.  (LDS has 64 banks = 256 bytes per clock: two 128-byte rows share
// a bank line, so 16 consecutive rows x one chunk must cover the 16 slots of a line.)
//
// Schedule.  With one wave per SIMD nothing hides an instruction clump, so the K loop is written
// as groups of {2 MFMAs, 1 LDS fragment read for the next K step, 1 tile load} pinned in source
// order: the matrix pipe keeps running while the other pipes are fed.  No branch sits inside the
// loop (each would make the register allocator shuffle the 256 accumulators).
//
// Epilogue.  The MFMA operands are swapped (weights as the row operand), so a lane holds 4
// consecutive output columns of one row; results are staged through LDS (free after the K loop)
// as bf16 and leave as 16-byte row-contiguous stores.  With SWIGLU the 128 B-rows of a wave's
// half tile are [gate c..c+31 | up c..c+31 | gate c+32..c+63 | up c+32..c+63], so MFMA row blocks
// (0,1) and (2,3) pair gate with up and the activation is applied in registers.
namespace t256 {
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int A_BYTES = BM * BK * 2;             // 32 KiB
constexpr int STAGE_BYTES = 2 * A_BYTES;         // 64 KiB: A tile then B tile
constexpr int EPI_STRIDE = 128 * 2 + 16;         // staged output row of a wave: 128 bf16 + pad
constexpr int EPI_BYTES = 4 * 128 * EPI_STRIDE;  // four waves x 128 rows
constexpr int SMEM_BYTES = EPI_BYTES > 2 * STAGE_BYTES ? EPI_BYTES : 2 * STAGE_BYTES;

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// 64 lanes x 16 bytes from global addresses base + off (base wave-uniform, off per lane, bytes)
// to LDS [lds, lds + 1024), asynchronously; completion is counted by vmcnt
__device__ __forceinline__ void load_to_lds_16(const char* base, unsigned off, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(off), "s"(base)
               : "memory", "m0");
}
#pragma clang diagnostic pop

// silu(g) * u with the hardware exp2 and reciprocal (about 1 ulp each: far inside bf16 rounding);
// the IEEE division would cost more VALU time per tile than the epilogue's stores
__device__ __forceinline__ float swiglu_fast(float g, float u) {
  const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
  return g * u * __builtin_amdgcn_rcpf(1.0f + e);
}

template <bool SWIGLU>
__global__ __launch_bounds__(256) void grouped_gemm_bf16(const GemmArgs a) {
  __shared__ __attribute__((aligned(1024))) char smem[SMEM_BYTES];
  __shared__ TileInfo s_info;

  constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
  const int n_tiles = (a.N + BN_OUT - 1) / BN_OUT;
  const TileMap tm = map_tile(n_tiles);
  const int n0 = tm.nt * BN_OUT;
  const TileInfo ti = find_tile<BM>(a, tm.mt, &s_info);
  if (ti.group < 0) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const long long widx = a.grp_widx ? a.grp_widx[ti.group] : (a.w_base + ti.group);

  // loader role: load i (0..7) of this wave fills tile rows (wave*8 + i)*8 .. +7 of A and of B;
  // lane -> row lane/8, slot lane%8
  unsigned a_off[8], b_off[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = (wave * 8 + i) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ ((r >> 1) & 7);
    int lr = ti.m0 + r;
    if (lr >= ti.rows) lr = ti.rows - 1;   // rows past the group are computed and dropped
    const int logical = ti.row_base + lr;
    const long long src = a.a_rows ? a.a_rows[logical] : logical;
    a_off[i] = (unsigned)((src * a.lda + chunk * 8) * 2);
    int ncol;
    if (SWIGLU) {
      const int half = r >> 7, q = (r & 127) >> 5, within = r & 31;
      ncol = n0 + half * 64 + (q >> 1) * 32 + within;   // q odd -> up matrix: loads 4..7 of every wave
    } else {
      ncol = n0 + r;
    }
    if (ncol >= a.N) ncol = a.N - 1;
    b_off[i] = (unsigned)(((long long)ncol * a.ldb + chunk * 8) * 2);
  }
  const char* a_base = static_cast<const char*>(a.A);
  const char* w_lo = static_cast<const char*>(a.B) + widx * a.b_group_stride * 2;                    // loads 0..3
  const char* w_hi = SWIGLU ? static_cast<const char*>(a.B2) + widx * a.b_group_stride * 2 : w_lo;   // loads 4..7
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
  const unsigned lds_w = __builtin_amdgcn_readfirstlane(lds0 + wave * 8192);

  // fragment read offsets inside a 32-row block for the four 16-wide K steps of a tile
  int foff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    foff[kk] = (lane & 31) * 128 + (((2 * kk + (lane >> 5)) ^ ((lane >> 1) & 7)) * 16);

  f32x16 acc[4][4];   // [weight-row block ni][token-row block mi]
#pragma unroll
  for (int ni = 0; ni < 4; ++ni)
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[ni][mi][r] = 0.0f;

  const int nk = a.K / BK;
  const int last = nk - 1;

  bf16x8 fa[2][4], fb[2][4];
  // fragment idx 0..3: token-row blocks, 4..7: weight-row blocks, of K step kk of the tile in `stage`
  auto read_frag = [&](int set, int stage, int kk, int idx) {
    const char* As = smem + stage * STAGE_BYTES + wm * 128 * 128;
    const char* Bs = smem + stage * STAGE_BYTES + A_BYTES + wn * 128 * 128;
    if (idx < 4)
      fa[set][idx] = *reinterpret_cast<const bf16x8*>(As + idx * 32 * 128 + foff[kk]);
    else
      fb[set][idx - 4] = *reinterpret_cast<const bf16x8*>(Bs + (idx - 4) * 32 * 128 + foff[kk]);
  };
  auto mfma_pair = [&](int set, int g) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int t = 2 * g + q, ni = t >> 2, mi = t & 3;
      acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][ni], fa[set][mi], acc[ni][mi], 0, 0, 0);
    }
  };
  // load g (0..7: A rows, 8..15: B rows) of K tile kt into `stage`.  Past the end the final tile
  // is fetched again into a stage nobody reads any more: keeps the loop free of branches.
  auto load_part = [&](int kt, int stage, int g) {
    const int kc = kt < nk ? kt : last;
    const int k0 = kc * BK;
    const unsigned lds = lds_w + stage * STAGE_BYTES;
    if (g < 8) {
      load_to_lds_16(a_base + (long long)k0 * 2, a_off[g], lds + g * 1024);
    } else {
      const int seg = k0 / a.kseg;   // which weight matrix along K (shared down projection)
      const long long kb = ((long long)seg * a.b_group_stride + (k0 - seg * a.kseg)) * 2;
      load_to_lds_16((g - 8 < 4 ? w_lo : w_hi) + kb, b_off[g - 8], lds + A_BYTES + (g - 8) * 1024);
    }
  };

  // prologue: tile 0 -> stage 0, its first fragments, first half of tile 1 -> stage 1
#pragma unroll
  for (int g = 0; g < 16; ++g) load_part(0, 0, g);
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
  for (int idx = 0; idx < 8; ++idx) read_frag(0, 0, 0, idx);
#pragma unroll
  for (int g = 0; g < 8; ++g) load_part(1, 1, g);
  __builtin_amdgcn_sched_barrier(0);

  // Steady state for tile kt in stage s: its step-0 fragments are in set 0, tile kt+1 is half
  // issued.  The block-wide wait for tile kt+1 sits before the last K step, so that the barrier
  // and the first fragment reads of tile kt+1 run under the 16 MFMAs of that step.
  for (int kt = 0; kt < nk; ++kt) {
    const int s = kt & 1;
    // K step 0: second half (B) of tile kt+1, fragments of step 1
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      load_part(kt + 1, s ^ 1, 8 + g);
      read_frag(1, s, 1, g);
      mfma_pair(0, g);
      __builtin_amdgcn_sched_barrier(0);
    }
    // K step 1: fragments of step 2
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      read_frag(0, s, 2, g);
      mfma_pair(1, g);
      __builtin_amdgcn_sched_barrier(0);
    }
    // K step 2: fragments of step 3
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      read_frag(1, s, 3, g);
      mfma_pair(0, g);
      __builtin_amdgcn_sched_barrier(0);
    }
    // tile kt+1 has landed (this wave's loads, then every wave's), and every wave has issued and
    // completed its last reads of stage s, which may therefore be refilled
    asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // K step 3: first half (A) of tile kt+2 -> stage s, step-0 fragments of tile kt+1
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      load_part(kt + 2, s, g);
      read_frag(0, s ^ 1, 0, g);
      mfma_pair(1, g);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // every load has landed and every wave has finished reading the stages: LDS is free for the epilogue
  asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

  // epilogue.  acc[ni][mi] element r of lane l: output row (token) mi*32 + l%32, output column
  // ni*32 + (r/4)*8 + (l/32)*4 + r%4 of the wave tile: 4 consecutive columns per register quad.
  char* stg = smem + wave * (128 * EPI_STRIDE);   // this wave's staging area, [128 rows][EPI_STRIDE]
  constexpr int W_COLS = SWIGLU ? 64 : 128;       // output columns of a wave tile
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    char* srow = stg + (mi * 32 + (lane & 31)) * EPI_STRIDE;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (SWIGLU) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          float h[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float g = acc[2 * p][mi][q * 4 + e], u = acc[2 * p + 1][mi][q * 4 + e];
            h[e] = swiglu_fast(g, u);
          }
          uint2 v;
          v.x = pack_bf16(h[0], h[1]);
          v.y = pack_bf16(h[2], h[3]);
          *reinterpret_cast<uint2*>(srow + (p * 32 + q * 8 + (lane >> 5) * 4) * 2) = v;
        }
      } else {
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
          uint2 v;
          v.x = pack_bf16(acc[ni][mi][q * 4 + 0], acc[ni][mi][q * 4 + 1]);
          v.y = pack_bf16(acc[ni][mi][q * 4 + 2], acc[ni][mi][q * 4 + 3]);
          *reinterpret_cast<uint2*>(srow + (ni * 32 + q * 8 + (lane >> 5) * 4) * 2) = v;
        }
      }
    }
  }
  // same wave reads back what it wrote: 16 bytes per lane along rows, row-contiguous global stores
  constexpr int CHUNKS = W_COLS / 8;              // 16-byte chunks per staged row
  constexpr int ROWS_PER_IT = 64 / CHUNKS;        // rows covered by one wave-wide access
  __bf16* C = static_cast<__bf16*>(a.C);
  const int col0 = n0 + wn * W_COLS + (lane % CHUNKS) * 8;
#pragma unroll 4
  for (int it = 0; it < 128 / ROWS_PER_IT; ++it) {
    const int rl = it * ROWS_PER_IT + lane / CHUNKS;          // row inside the wave tile
    const int row = ti.m0 + wm * 128 + rl;
    const u32x4 v = *reinterpret_cast<const u32x4*>(stg + rl * EPI_STRIDE + (lane % CHUNKS) * 16);
    if (row < ti.rows && col0 < a.N)
      *reinterpret_cast<u32x4*>(C + (long long)(ti.row_base + row) * a.ldc + a.c_col0 + col0) = v;
  }
}
}  // namespace t256

// ------------------------------------------------------------------------------------------
// f32 kernel: 16 x 16 outputs per block, one output per thread, 16-wide K slices through LDS.
constexpr int FM = 16, FN = 16, FK = 16;

template <bool SWIGLU>
__global__ __launch_bounds__(FM * FN) void grouped_gemm_f32(const GemmArgs a) {
  __shared__ float As[FM][FK + 1], Bs[FN][FK + 1], B2s[FN][FK + 1];
  __shared__ TileInfo s_info;
  const int n_tiles = (a.N + FN - 1) / FN;
  const int mt = blockIdx.x / n_tiles;
  const int n0 = (blockIdx.x % n_tiles) * FN;
  const TileInfo ti = find_tile<FM>(a, mt, &s_info);
  if (ti.group < 0) return;
  const int tx = threadIdx.x % FN, ty = threadIdx.x / FN;
  const float* A = static_cast<const float*>(a.A);
  const long long widx = a.grp_widx ? a.grp_widx[ti.group] : (a.w_base + ti.group);

  // loader roles: thread (ty, tx) loads A[row ty][k tx] and B[col ty][k tx]
  int lr = ti.m0 + ty;
  if (lr >= ti.rows) lr = ti.rows - 1;
  const int logical = ti.row_base + lr;
  const long long src = a.a_rows ? a.a_rows[logical] : logical;
  const float* a_row = A + src * a.lda;
  int ncol = n0 + ty;
  if (ncol >= a.N) ncol = a.N - 1;
  const float* b_row = static_cast<const float*>(a.B) + widx * a.b_group_stride + (long long)ncol * a.ldb;
  const float* b2_row =
      SWIGLU ? static_cast<const float*>(a.B2) + widx * a.b_group_stride + (long long)ncol * a.ldb : nullptr;

  float acc = 0.0f, acc2 = 0.0f;
  for (int k0 = 0; k0 < a.K; k0 += FK) {
    const int kk = k0 + tx;
    const int seg = kk / a.kseg;
    const long long boff = (long long)seg * a.b_group_stride + (kk - seg * a.kseg);
    As[ty][tx] = (kk < a.K) ? a_row[kk] : 0.0f;
    Bs[ty][tx] = (kk < a.K) ? b_row[boff] : 0.0f;
    if (SWIGLU) B2s[ty][tx] = (kk < a.K) ? b2_row[boff] : 0.0f;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < FK; ++q) {
      acc = fmaf(As[ty][q], Bs[tx][q], acc);
      if (SWIGLU) acc2 = fmaf(As[ty][q], B2s[tx][q], acc2);
    }
    __syncthreads();
  }
  const int row = ti.m0 + ty, col = n0 + tx;
  if (row < ti.rows && col < a.N) {
    float* C = static_cast<float*>(a.C);
    const float out = SWIGLU ? acc / (1.0f + expf(-acc)) * acc2 : acc;
    C[(long long)(ti.row_base + row) * a.ldc + a.c_col0 + col] = out;
  }
}

static int launch_gemm(const occult_cfg_t& c, const GemmArgs& a, bool swiglu, int total_rows, hipStream_t s) {
  if (total_rows == 0) return OCCULT_OK;
  if (c.dtype == OCCULT_BF16) {
    // rows per group decide the tile: 256-row tiles once groups average >= 192 rows
    const int groups = a.grp_offset ? a.ngroups : 1;
    // 256-row tiles once groups average >= 192 rows and every A byte offset fits 32 bits
    const bool use_big = (long long)total_rows >= 192ll * groups &&
                         (long long)a.a_rows_total * a.lda * 2 < (1ll << 32);
    const int bm = use_big ? t256::BM : small::BM;
    const int bn = use_big ? t256::BN : small::BN;
    const int bn_out = swiglu ? bn / 2 : bn;
    const long long m_tiles = (total_rows + bm - 1) / bm + (a.grp_offset ? a.ngroups : 0);
    const long long blocks = mapped_grid(m_tiles, (a.N + bn_out - 1) / bn_out);
    OCC_REQUIRE(blocks < (1ll << 31), OCCULT_EINVAL, "grouped GEMM grid too large");
    const dim3 grid((unsigned)blocks), block(256);
    if (use_big) {
      if (swiglu) hipLaunchKernelGGL(t256::grouped_gemm_bf16<true>, grid, block, 0, s, a);
      else hipLaunchKernelGGL(t256::grouped_gemm_bf16<false>, grid, block, 0, s, a);
    } else {
      if (swiglu) hipLaunchKernelGGL(small::grouped_gemm_bf16<true>, grid, block, 0, s, a);
      else hipLaunchKernelGGL(small::grouped_gemm_bf16<false>, grid, block, 0, s, a);
    }
  } else {
    const long long m_tiles = (total_rows + FM - 1) / FM + (a.grp_offset ? a.ngroups : 0);
    const long long blocks = m_tiles * ((a.N + FN - 1) / FN);
    OCC_REQUIRE(blocks < (1ll << 31), OCCULT_EINVAL, "grouped GEMM grid too large");
    if (swiglu)
      hipLaunchKernelGGL(grouped_gemm_f32<true>, dim3((unsigned)blocks), dim3(FM * FN), 0, s, a);
    else
      hipLaunchKernelGGL(grouped_gemm_f32<false>, dim3((unsigned)blocks), dim3(FM * FN), 0, s, a);
  }
  OCC_LAUNCH_CHECK("grouped_gemm");
  return OCCULT_OK;
}

}  // namespace occult

using namespace occult;

extern "C" int occult_expert_ffn(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                 const void* x, const occult_weights_t* weights, void* epd_h, void* epd_y,
                                 void* h_shared, void* y_shared, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(plan && plan->exp_offset && plan->pos_expert && plan->epd_sfd_row, OCCULT_ENULLPTR,
              "plan or one of its tables is NULL");
  OCC_REQUIRE(weights && weights->w_gate && weights->w_up && weights->w_down, OCCULT_ENULLPTR,
              "weights or one of its tensors is NULL");
  OCC_REQUIRE(sfd_x && epd_h && epd_y, OCCULT_ENULLPTR, "sfd_x, epd_h or epd_y is NULL");
  if (c.S > 0)
    OCC_REQUIRE(x && h_shared && y_shared, OCCULT_ENULLPTR, "x, h_shared or y_shared is NULL with S=%d", c.S);
  const int es = elem_size(c);
  OCC_REQUIRE(((size_t)c.d * es) % 16 == 0 && ((size_t)c.f * es) % 16 == 0, OCCULT_EALIGN,
              "rows of d=%d or f=%d elements are not multiples of 16 bytes", c.d, c.f);
  if (c.dtype == OCCULT_BF16)
    OCC_REQUIRE(c.d % 64 == 0 && c.f % 64 == 0, OCCULT_ESHAPE,
                "bf16 path needs d and f to be multiples of 64 (d=%d, f=%d)", c.d, c.f);
  OCC_REQUIRE(aligned16(sfd_x) && aligned16(epd_h) && aligned16(epd_y) && aligned16(x) &&
                  aligned16(h_shared) && aligned16(y_shared) && aligned16(weights->w_gate) &&
                  aligned16(weights->w_up) && aligned16(weights->w_down),
              OCCULT_EALIGN, "a buffer is not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n_epd = c.T * c.k;

  GemmArgs g1{};
  g1.A = sfd_x; g1.lda = c.d; g1.a_rows = plan->epd_sfd_row;
  g1.B = weights->w_gate; g1.B2 = weights->w_up;
  g1.b_group_stride = (long long)c.f * c.d; g1.ldb = c.d; g1.kseg = c.d;
  g1.C = epd_h; g1.ldc = c.f; g1.c_col0 = 0;
  g1.grp_offset = plan->exp_offset; g1.grp_widx = plan->pos_expert; g1.w_base = 0;
  g1.ngroups = c.E; g1.M = 0; g1.N = c.f; g1.K = c.d;
  g1.a_rows_total = sfd_rows_max(c);
  const bool do1 = c.ffn_phase != 2, do2 = c.ffn_phase != 1;
  if (do1) {
    rc = launch_gemm(c, g1, true, n_epd, s);
    if (rc) return rc;
  }

  GemmArgs g2{};
  g2.A = epd_h; g2.lda = c.f; g2.a_rows = nullptr;
  g2.B = weights->w_down; g2.B2 = nullptr;
  g2.b_group_stride = (long long)c.d * c.f; g2.ldb = c.f; g2.kseg = c.f;
  g2.C = epd_y; g2.ldc = c.d; g2.c_col0 = 0;
  g2.grp_offset = plan->exp_offset; g2.grp_widx = plan->pos_expert; g2.w_base = 0;
  g2.ngroups = c.E; g2.M = 0; g2.N = c.d; g2.K = c.f;
  g2.a_rows_total = n_epd;
  if (do2) {
    rc = launch_gemm(c, g2, false, n_epd, s);
    if (rc) return rc;
  }

  if (c.S > 0) {
    // shared experts: h_shared[t][s*f .. (s+1)*f) per shared expert, then one product whose K
    // dimension walks the S down-projection matrices
    for (int sh = 0; do1 && sh < c.S; ++sh) {
      GemmArgs a1{};
      a1.A = x; a1.lda = c.d; a1.a_rows = nullptr;
      a1.B = weights->w_gate; a1.B2 = weights->w_up;
      a1.b_group_stride = (long long)c.f * c.d; a1.ldb = c.d; a1.kseg = c.d;
      a1.C = h_shared; a1.ldc = c.S * c.f; a1.c_col0 = sh * c.f;
      a1.grp_offset = nullptr; a1.grp_widx = nullptr; a1.w_base = c.E + sh;
      a1.ngroups = 1; a1.M = c.T; a1.N = c.f; a1.K = c.d; a1.a_rows_total = c.T;
      rc = launch_gemm(c, a1, true, c.T, s);
      if (rc) return rc;
    }
    GemmArgs a2{};
    a2.A = h_shared; a2.lda = c.S * c.f; a2.a_rows = nullptr;
    a2.B = weights->w_down; a2.B2 = nullptr;
    a2.b_group_stride = (long long)c.d * c.f; a2.ldb = c.f; a2.kseg = c.f;
    a2.C = y_shared; a2.ldc = c.d; a2.c_col0 = 0;
    a2.grp_offset = nullptr; a2.grp_widx = nullptr; a2.w_base = c.E;
    a2.ngroups = 1; a2.M = c.T; a2.N = c.d; a2.K = c.S * c.f; a2.a_rows_total = c.T;
    if (do2) {
      rc = launch_gemm(c, a2, false, c.T, s);
      if (rc) return rc;
    }
  }
  return OCCULT_OK;
}
