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
#include "gemm.h"

#include <type_traits>

namespace occult {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct TileInfo {
  int group, m0, rows, row_base;
};
// first output column of a group
__device__ __forceinline__ int group_col0(const GemmArgs& a, int group) { return a.c_col0 + group * a.c_group_cols; }

// Workgroup id -> (m-tile, n-tile).  Workgroups are handed to the 8 XCDs round-robin and each XCD
// has its own L2, so the tiles an XCD runs at the same time should share operands: XCD x gets
// "chunks" x, x+8, ... of MC consecutive m-tiles times all n-tiles (about one tile per CU of the
// XCD), so that an A tile is fetched into one L2 only and a B tile is reused MC times there.
struct TileMap {
  int mt, nt;
};
__device__ __forceinline__ TileMap map_tile_id(unsigned b, int n_tiles) {
  const int mc = max(1, (32 + n_tiles / 2) / n_tiles);
  const unsigned per_chunk = mc * n_tiles;
  const int xcd = (int)(b & 7);
  const unsigned slot = b >> 3;
  const int chunk = (int)(slot / per_chunk) * 8 + xcd;
  const int within = (int)(slot % per_chunk);
  TileMap tm;
  tm.mt = chunk * mc + within / n_tiles;
  tm.nt = within % n_tiles;
  return tm;
}
__device__ __forceinline__ TileMap map_tile(int n_tiles) { return map_tile_id(blockIdx.x, n_tiles); }
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
      const int per_group = (a.M + BM - 1) / BM;
      if (mt < per_group * a.ngroups) {
        ti.group = mt / per_group;
        ti.m0 = (mt % per_group) * BM;
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
  __shared__ __attribute__((aligned(16))) __bf16 As[2][BM * LDS_STRIDE];   // two K tiles: one multiplied, one being written
  __shared__ __attribute__((aligned(16))) __bf16 Bs[2][BN * LDS_STRIDE];
  __shared__ TileInfo s_info;

  constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
  const int n_tiles = (a.N + BN_OUT - 1) / BN_OUT;
  TileMap tm = map_tile(n_tiles);
  if (a.plain_map) {
    tm.mt = blockIdx.x / n_tiles;
    tm.nt = blockIdx.x % n_tiles;
  }
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

  const int nk_all = a.K / BK;
  const int split = a.ksplit > 1 ? a.ksplit : 1;
  const int kt_begin = (int)((long long)blockIdx.y * nk_all / split);   // this block's K tiles
  const int nk = (int)((long long)(blockIdx.y + 1) * nk_all / split);   // (end, exclusive)
  // A block is alone on its CU more often than not (few tiles), so nothing else hides its own latencies: the
  // K loop is software-pipelined.  While K tile kt is multiplied out of one LDS buffer, tile kt+1 (already in
  // registers) is written to the other, tile kt+2 is in flight into the second register set and tile kt+3 is
  // requested as soon as a set is free; inside a tile the fragments of K step kk+1 are read while step kk is
  // multiplied; one barrier per tile.
  u32x4 ga0[4], gb0[4], ga1[4], gb1[4];
  auto load_global = [&](int kt, u32x4 (&ga)[4], u32x4 (&gb)[4]) {
    const int k0 = kt * BK;
    const int seg = k0 / a.kseg;                 // which weight matrix along K (shared down-proj)
    const long long boff = (long long)seg * a.b_group_stride + (k0 - seg * a.kseg);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ga[i] = *reinterpret_cast<const u32x4*>(a_src[i] + k0);
      gb[i] = *reinterpret_cast<const u32x4*>(b_src[i] + boff);
    }
  };
  auto write_lds = [&](int buf, const u32x4 (&ga)[4], const u32x4 (&gb)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = r_in + 32 * i;
      *reinterpret_cast<u32x4*>(&As[buf][r * LDS_STRIDE + kv * 8]) = ga[i];
      *reinterpret_cast<u32x4*>(&Bs[buf][r * LDS_STRIDE + kv * 8]) = gb[i];
    }
  };
  bf16x8 fa[2][2], fb[2][2];
  auto read_frags = [&](int buf, int kk, bf16x8 (&xa)[2], bf16x8 (&xb)[2]) {
    const int kof = kk * 16 + (lane >> 5) * 8;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
      xa[mi] = *reinterpret_cast<const bf16x8*>(&As[buf][(wm * 64 + mi * 32 + (lane & 31)) * LDS_STRIDE + kof]);
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
      xb[ni] = *reinterpret_cast<const bf16x8*>(&Bs[buf][(wn * 64 + ni * 32 + (lane & 31)) * LDS_STRIDE + kof]);
  };
  // K tile kt out of LDS buffer `buf`; (ga, gb) holds tile kt+1 on entry and is refilled with tile kt+3
  auto k_tile = [&](int kt, int buf, u32x4 (&ga)[4], u32x4 (&gb)[4]) {
    read_frags(buf, 0, fa[0], fb[0]);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) read_frags(buf, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
      if (kk == 1 && kt + 1 < nk) write_lds(buf ^ 1, ga, gb);
      if (kk == 2 && kt + 3 < nk) load_global(kt + 3, ga, gb);
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][mi], fb[kk & 1][ni], acc[mi][ni], 0, 0, 0);
    }
    __syncthreads();   // tile kt+1 is in the other buffer for everyone, and nobody reads this one any more
  };
  if (kt_begin < nk) {
    load_global(kt_begin, ga0, gb0);
    if (kt_begin + 1 < nk) load_global(kt_begin + 1, ga1, gb1);
    write_lds(0, ga0, gb0);
    if (kt_begin + 2 < nk) load_global(kt_begin + 2, ga0, gb0);
    __syncthreads();
    for (int kt = kt_begin; kt < nk; kt += 2) {
      k_tile(kt, 0, ga1, gb1);
      if (kt + 1 < nk) k_tile(kt + 1, 1, ga0, gb0);
    }
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
      __bf16* crow = C + (long long)(ti.row_base + row) * a.ldc + group_col0(a, ti.group);
      if (!SWIGLU && a.ksplit > 1) {   // partial sums of this K slice, f32
        float* prow = a.ws + ((long long)blockIdx.y * a.M + row) * a.N;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          const int col = n0 + wn * 64 + ni * 32 + col_in;
          if (col < a.N) prow[col] = acc[mi][ni][r];
        }
        continue;
      }
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
// bf16 MFMA kernel for groups of a few rows (decode-shaped layers), where the work is streaming
// every active expert's weights from HBM once.  No LDS tiles, no barriers in the K loop: each wave
// owns 32 output columns x up to 16*MT tokens over the whole K (or a quarter of it: KSPLIT below)
// and loads both operands straight into MFMA fragment registers.  v_mfma_f32_16x16x32_bf16 takes 8 consecutive K elements per lane
// and 4 lanes per row, so one load instruction reads 16 rows x one whole 64-byte sector.  Weights
// are the row operand: a lane ends up with 4 consecutive output columns of one token (8-byte
// stores).  The operands of the next K step (4 or 8 KiB of weights per wave) are in flight while
// the current ones are multiplied; token blocks past the group's rows are skipped.
//
// One launch can carry two problems of the same shape class (N, SWIGLU, weight order): workgroups
// [0, a_blocks) work on `first`, the rest on `second`.  A small batch's shared experts ride with its
// routed experts this way: alone their few workgroups would stream weights at a fraction of the memory
// system's rate, and run after the routed experts they would add their whole duration to the call.
// The second problem has uniform groups and always splits K over the four waves of a workgroup (below);
// its K may walk several weight matrices (the shared experts' down projection: K = S * f), so that
// the sum over the shared experts happens in the accumulators and in the in-LDS addition, in K order.
namespace skinny {
constexpr int BN_OUT = 32;
typedef float f32x4v __attribute__((ext_vector_type(4)));

// KSPLIT (for the first problem; the second always does): the four waves of a workgroup take the four quarters of K
// of ONE column block and add their sums through LDS (quarters in ascending order, so the result is reproducible)
// instead of taking four column blocks over the whole K.  A wave's stream is then a quarter as long and there are four times as many workgroups, which the
// hardware hands to whichever CU has room: with whole-K waves a layer's 2000-4000 waves fill the chip's 1024 SIMDs
// two to four deep, all finish together, and a last partly filled layer of waves costs a whole stream's time.
template <bool SWIGLU, int MT, bool PACKED, bool KSPLIT>   // MT token blocks of 16 per m-tile; PACKED: weights from a.Bp
__global__ __launch_bounds__(256) void grouped_gemm_bf16(const GemmArgs first, const GemmArgs second, const int a_blocks) {
  constexpr int BM = 16 * MT;
  constexpr int KS = MT <= 2 ? 2 : 1;   // 32-wide K steps per pipeline stage
  constexpr int NW = SWIGLU ? 2 : 1;
  static_assert(!PACKED || KS == 2, "the packed order is written for two K steps per stage");
  __shared__ TileInfo s_info;
  const bool is_second = (int)blockIdx.x >= a_blocks;   // uniform over the workgroup
  const GemmArgs& a = is_second ? second : first;
  const bool ksplit = KSPLIT || is_second;   // uniform: the second problem's workgroups always split K
  const int cbw = ksplit ? 1 : 4;            // column blocks per workgroup
  const int n_cb = a.N / BN_OUT;   // column blocks (host: N % 32 == 0)
  const int wgs_per_mt = (n_cb + cbw - 1) / cbw;
  int mt, cbq;   // m-tile and group of cbw column blocks
  if (!is_second) {
    mt = (int)blockIdx.x / wgs_per_mt;
    cbq = (int)blockIdx.x % wgs_per_mt;
  } else {
    // Uniform groups of P m-tiles each: the P workgroups that stream the same weights (one per m-tile) get ids
    // 8 apart, so they run on the same XCD (workgroups go to the 8 XCDs round-robin) at about the same time and
    // all but the first of them find the weights in that XCD's L2.  unit = (group, column block).
    // (Measured against the four waves of one workgroup taking the m-tiles of one column block, which shares
    // the weights inside a CU: that was slower from 64 tokens on.)
    const int b = (int)blockIdx.x - a_blocks;
    const int P = (a.M + BM - 1) / BM;
    const int unit = b / (8 * P) * 8 + (b & 7), m = (b >> 3) % P;
    if (unit >= a.ngroups * wgs_per_mt) return;   // uniform: the grid is padded to whole sets of 8 units
    mt = unit / wgs_per_mt * P + m;
    cbq = unit % wgs_per_mt;
  }
  TileInfo ti = find_tile<BM>(a, mt, &s_info);
  if (ti.group < 0) return;
  // what came through LDS is the same in every lane: kept in scalar registers, so that the addresses built from it
  // are a scalar base plus a per-lane 32-bit offset
  ti.group = __builtin_amdgcn_readfirstlane(ti.group);
  ti.m0 = __builtin_amdgcn_readfirstlane(ti.m0);
  ti.rows = __builtin_amdgcn_readfirstlane(ti.rows);
  ti.row_base = __builtin_amdgcn_readfirstlane(ti.row_base);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int cb = ksplit ? cbq : cbq * 4 + wave;
  if (cb >= n_cb) return;   // whole-K workgroups meet no barrier after this; K-splitting ones never take it
  const int n0 = cb * BN_OUT;
  const int r = lane & 15, c = lane >> 4;
  const long long widx = __builtin_amdgcn_readfirstlane(a.grp_widx ? a.grp_widx[ti.group] : (a.w_base + ti.group));
  const int nblk = min(MT, (ti.rows - ti.m0 + 15) / 16);   // token blocks with any valid row
  const bool reread = is_second && a.M > BM;   // uniform

  // this lane's weight rows (column blocks 0 and 1 of the unit) and token rows, at its 16-byte K group
  const char* w[NW][2];
#pragma unroll
  for (int m = 0; m < NW; ++m)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
      w[m][nb] = static_cast<const char*>(m == 0 ? a.B : a.B2) +   // loaded like the token rows: lane l on row l / 4
                 ((widx * a.b_group_stride + (long long)(n0 + nb * 16 + (lane >> 2)) * a.ldb) * 2 + (lane & 3) * 16);
  // packed order: this wave's unit is one contiguous stream of stages, a load instruction reads 1 KiB of it
  const long long unit_bytes = (long long)(BN_OUT * NW * 2) * a.kseg;   // one unit's stream inside one weight matrix
  const char* wp = PACKED ? static_cast<const char*>(a.Bp) + widx * a.bp_group_stride + cb * unit_bytes
                          : nullptr;   // scalar; a lane reads at lane * 16 from it
  const unsigned lane16 = lane * 16;
  // token rows: a scalar base plus a 32-bit byte offset per lane (host: A < 4 GiB).  The MFMA wants lane l to hold row
  // l % 16, K group l / 16, which would make neighbouring lanes read rows that lie a whole row pitch apart (16 cache
  // lines looked up per 16 lanes).  The rows are loaded instead with lane l on row l / 4, K group l % 4 (four
  // neighbouring lanes = one 64-byte sector, 4 lines per 16 lanes) and put into the MFMA's order by a lane permutation
  // just before use (ds_bpermute: the LDS crossbar, no LDS memory).
  const char* xbase = static_cast<const char*>(a.A);
  unsigned xo[MT];
#pragma unroll
  for (int tb = 0; tb < MT; ++tb) {
    int lr = ti.m0 + tb * 16 + (lane >> 2);
    if (lr >= ti.rows) lr = ti.rows - 1;   // tokens past the group's end repeat its last row; dropped at the end
    const int logical = ti.row_base + lr;
    const unsigned src = a.a_rows ? a.a_rows[logical] : logical;
    xo[tb] = (src * (unsigned)a.lda) * 2u + (lane & 3) * 16;
  }
  const int from_lane4 = (r * 4 + c) * 4;   // byte index of the lane that loaded what this lane multiplies
  auto to_mfma_order = [&](const bf16x8& v) {
    typedef int i32x4v __attribute__((ext_vector_type(4)));
    i32x4v t = __builtin_bit_cast(i32x4v, v);
#pragma unroll
    for (int e = 0; e < 4; ++e) t[e] = __builtin_amdgcn_ds_bpermute(from_lane4, t[e]);
    return __builtin_bit_cast(bf16x8, t);
  };

  f32x4v acc[NW][2][MT];
#pragma unroll
  for (int m = 0; m < NW; ++m)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int tb = 0; tb < MT; ++tb) acc[m][nb][tb] = f32x4v{0.0f, 0.0f, 0.0f, 0.0f};

  const int nst = a.K / (32 * KS);   // pipeline stages along K (host: K % 64 == 0)
  // byte offset of the current stage inside a weight row; K > kseg walks consecutive weight matrices
  long long w_off = 0, p_off = 0;   // caller's layout / packed order
  int w_kin = 0;
  auto w_advance = [&]() {
    w_off += 64 * KS;
    p_off += KS * NW * 2048;
    w_kin += 32 * KS;
    if (w_kin >= a.kseg) {   // host: kseg % 64 == 0, so a stage never straddles two matrices
      w_kin = 0;
      w_off += (a.b_group_stride - a.kseg) * 2;
      p_off += a.bp_group_stride - unit_bytes;
    }
  };
  struct Stage {
    bf16x8 wf[KS][NW][2], xf[KS][MT];
  };
  auto load_stage = [&](Stage& st, long long woff, long long poff, int i) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int m = 0; m < NW; ++m)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          {
            // measured: the streaming hint helps the single-matrix product and hurts the gate/up pair
            const bf16x8* src = PACKED ? reinterpret_cast<const bf16x8*>(wp + (poff + ((ks * NW + m) * 2 + nb) * 1024) +
                                                                           (size_t)lane16)
                                       : reinterpret_cast<const bf16x8*>(w[m][nb] + woff + ks * 64);
            // (a problem whose groups span several m-tiles reads its weights once per m-tile: those stay cacheable)
            st.wf[ks][m][nb] = (SWIGLU || reread) ? *src : __builtin_nontemporal_load(src);
          }
#pragma unroll
      for (int tb = 0; tb < MT; ++tb)
        if (tb < nblk) st.xf[ks][tb] = *reinterpret_cast<const bf16x8*>(xbase + ((long long)i * KS + ks) * 64 + (size_t)xo[tb]);
    }
  };
  auto multiply = [&](const Stage& st) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 wfo[NW][2];   // the packed order is the MFMA's already
#pragma unroll
      for (int m = 0; m < NW; ++m)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) wfo[m][nb] = PACKED ? st.wf[ks][m][nb] : to_mfma_order(st.wf[ks][m][nb]);
#pragma unroll
      for (int tb = 0; tb < MT; ++tb)
        if (tb < nblk) {
          const bf16x8 xf = to_mfma_order(st.xf[ks][tb]);
#pragma unroll
          for (int m = 0; m < NW; ++m)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
              acc[m][nb][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfo[m][nb], xf, acc[m][nb][tb], 0, 0, 0);
        }
    }
  };

  // this wave's stages of K
  const int i_begin = ksplit ? wave * nst / 4 : 0, i_end = ksplit ? (wave + 1) * nst / 4 : nst;
  if (i_begin > 0) {
    const int kin = i_begin * 32 * KS, mat = kin / a.kseg;
    w_kin = kin - mat * a.kseg;
    w_off = ((long long)mat * a.b_group_stride + w_kin) * 2;
    p_off = mat * a.bp_group_stride + (long long)(w_kin / 32) * (NW * 2048);
  }
  if (i_begin < i_end) {   // wave-uniform
    Stage s0, s1;
    load_stage(s0, w_off, p_off, i_begin);
    for (int i = i_begin; i < i_end; i += 2) {
      // past the end the last stage is fetched again and not used
      const bool more1 = i + 1 < i_end;
      if (more1) w_advance();
      load_stage(s1, w_off, p_off, more1 ? i + 1 : i);
      multiply(s0);
      const bool more2 = i + 2 < i_end;
      if (more2) w_advance();
      load_stage(s0, w_off, p_off, more2 ? i + 2 : (more1 ? i + 1 : i));
      if (more1) multiply(s1);
    }
  }
  if (ksplit) {   // uniform over the workgroup
    // waves 1..3 hand their sums to wave 0, which adds them in that order and writes the tile
    __shared__ float s_red[3][NW * 2 * MT * 4][64];
    if (wave > 0) {
#pragma unroll
      for (int m = 0; m < NW; ++m)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int tb = 0; tb < MT; ++tb)
#pragma unroll
            for (int e = 0; e < 4; ++e) s_red[wave - 1][((m * 2 + nb) * MT + tb) * 4 + e][lane] = acc[m][nb][tb][e];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int wv = 0; wv < 3; ++wv)
#pragma unroll
      for (int m = 0; m < NW; ++m)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int tb = 0; tb < MT; ++tb)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[m][nb][tb][e] += s_red[wv][((m * 2 + nb) * MT + tb) * 4 + e][lane];
  }

  // acc element e of lane l: token l%16 of its block, output column nb*16 + (l/16)*4 + e of the unit
#pragma unroll
  for (int tb = 0; tb < MT; ++tb) {
    const int token = ti.m0 + tb * 16 + r;
    if (token < ti.rows) {
      __bf16* crow = static_cast<__bf16*>(a.C) + (long long)(ti.row_base + token) * a.ldc + group_col0(a, ti.group) + n0 + c * 4;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float g = acc[0][nb][tb][e];
          v[e] = SWIGLU ? g / (1.0f + __expf(-g)) * acc[NW - 1][nb][tb][e] : g;
        }
        uint2 pk;
        pk.x = pack_bf16(v[0], v[1]);
        pk.y = pack_bf16(v[2], v[3]);
        *reinterpret_cast<uint2*>(crow + nb * 16) = pk;
      }
    }
  }
}
}  // namespace skinny

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel, main variant (prefill-shaped layers).  Block = 256 threads = 4 waves (2 x 2),
// block tile 256 x 256 x 64, wave tile 128 x 128 = 4 x 4 MFMA tiles of 32 x 32 (256 accumulator
// registers per lane, one wave per SIMD, one block per CU).
//
// Persistent blocks.  With one block per CU nothing overlaps a tile's fixed costs (finding its
// group, gathering its row indices, the first operand loads, the store tail), so a block walks
// output tiles blockIdx.x, + gridDim.x, ... of the XCD-aware order and treats them as one stream
// of K tiles: the next output tile's group and row gather are fetched during the current K loop,
// its first K tile is loaded during the current tile's last two K tiles, and its second one
// during the epilogue.
//
// Global -> LDS.  Operand tiles go from global memory straight into LDS
// (global_load_lds_dwordx4: no VGPR staging, no ds_write), double buffered: while K tile j is
// multiplied, K tile j+1 lands in the other stage.  The loads are issued from inline assembly
// (wave-uniform base in SGPRs + a 32-bit per-lane offset that is constant over K, so advancing K
// costs two scalar adds) and waited for with an explicit vmcnt: the compiler's own wait insertion
// treats an LDS-directed load as a FLAT access and could only wait for all outstanding loads at
// every LDS read.  One such load writes 64 lanes x 16 bytes contiguously = 8 rows of 128 bytes,
// so rows cannot be padded; bank conflicts of the 16-byte fragment reads are avoided by an XOR
// swizzle instead: chunk c of row r lives at slot c ^ ((r >> 1) & 7), realised by the loading
// lane's choice of global chunk.  (LDS has 64 banks = 256 bytes per clock: two 128-byte rows share
// a bank line, so 16 consecutive rows x one chunk must cover the 16 slots of a line.)
//
// Schedule.  With one wave per SIMD nothing hides an instruction clump, so a K step (16 MFMAs) is
// written as 8 groups of {2 MFMAs, 1 LDS fragment read for the next K step, 1 tile load} pinned in
// source order: the matrix pipe keeps running while the other pipes are fed.  The steps of a K
// tile are rotated to 1, 2, wait, 3, 0': the block-wide wait for the next K tile sits before step
// 3, so the barrier and the first fragment reads of that tile run under 16 MFMAs.  Step 0 of an
// output tile multiplies into a zero constant, so accumulators are never cleared.  No branch sits
// inside a K tile (each would make the register allocator shuffle the 256 accumulators).
//
// Epilogue.  The MFMA operands are swapped (weights as the row operand), so a lane holds 4
// consecutive output columns of one row; results go as bf16 through the wave's own 8 KiB of the
// idle stage (the region its own next loads will fill, so no block barrier is needed), 32 rows x
// 64 columns at a time, and leave as 16-byte stores of whole 128-byte row segments.  With SWIGLU
// the 128 B-rows of a wave's half tile are [gate c..c+31 | up c..c+31 | gate c+32..c+63 |
// up c+32..c+63], so MFMA row blocks (0,1) and (2,3) pair gate with up and the activation is
// applied in registers.
namespace t256 {
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int A_BYTES = BM * BK * 2;             // 32 KiB
constexpr int STAGE_BYTES = 2 * A_BYTES;         // 64 KiB: A tile then B tile
constexpr int SMEM_BYTES = 2 * STAGE_BYTES;

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// 64 lanes x 16 bytes from global addresses base + off (base wave-uniform, off per lane, bytes)
// to LDS [lds, lds + 1024), asynchronously; completion is counted by vmcnt
__device__ __forceinline__ void load_to_lds_16(const char* base, unsigned off, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(off), "s"(base)
               : "memory", "m0");
}
// the same from one 64-bit address per lane
__device__ __forceinline__ void load_to_lds_16(const char* src, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(src) : "memory", "m0");
}
// every load of this wave has landed and its LDS reads have returned; then the same for the block
__device__ __forceinline__ void wait_all_and_barrier() {
  asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
#pragma clang diagnostic pop

// silu(g) * u with the hardware exp2 and reciprocal (about 1 ulp each: far inside bf16 rounding);
// the IEEE division would cost more VALU time per tile than the epilogue's stores
__device__ __forceinline__ float swiglu_fast(float g, float u) {
  const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
  return g * u * __builtin_amdgcn_rcpf(1.0f + e);
}

// One output tile before its row gather has come back.  All fields but raw are wave-uniform.
struct Head {
  int valid, m0, rows, row_base, n0, widx, ccol;   // ccol: first output column of the tile's group
  int raw[8];   // source rows of this lane's 8 A-tile rows
};

// which group and row block is m-tile mt?  s_tpre[g] = m-tiles of the groups before g (s_tpre[ngroups]
// = all of them).  Every wave works this out for itself; the result is wave-uniform.
// group = -1: past the last tile.
__device__ __forceinline__ void locate(const GemmArgs& a, const int* s_goff, const int* s_tpre, int mt, int lane,
                                       int& group, int& m0, int& rows, int& row_base) {
  group = -1;
  m0 = rows = row_base = 0;
  if (a.grp_offset == nullptr) {
    const int per_group = (a.M + BM - 1) / BM;
    if (mt < per_group * a.ngroups) {
      group = mt / per_group;
      m0 = (mt % per_group) * BM;
      rows = a.M;
    }
    return;
  }
  for (int c0 = 0; c0 < a.ngroups; c0 += 64) {
    const int g = c0 + lane;
    const bool mine = g < a.ngroups && mt >= s_tpre[g] && mt < s_tpre[g + 1];
    const unsigned long long hit = __ballot(mine);
    if (hit) {   // wave-uniform
      group = c0 + __ffsll((long long)hit) - 1;
      m0 = (mt - s_tpre[group]) * BM;
      row_base = s_goff[group];
      rows = s_goff[group + 1] - row_base;
      return;
    }
  }
}


// SAVE (with SWIGLU): the gate and up pre-activations are stored too (a.C2).
// WIDE: the A operand is 4 GiB or larger, so its per-lane byte offsets take 64 bits (two registers per load
// and a 64-bit add before each) instead of one 32-bit offset beside a scalar base.
template <bool SWIGLU, bool SAVE, bool WIDE = false>
__global__ __launch_bounds__(256) void grouped_gemm_bf16(const GemmArgs a) {
  static_assert(SWIGLU || !SAVE, "pre-activations exist only with the fused activation");
  using aoff_t = typename std::conditional<WIDE, unsigned long long, unsigned>::type;
  __shared__ __attribute__((aligned(1024))) char smem[SMEM_BYTES];
  __shared__ int s_goff[OCCULT_MAX_E + 1];   // group row offsets
  __shared__ int s_widx[OCCULT_MAX_E];       // weight matrix of each group
  __shared__ int s_tpre[OCCULT_MAX_E + 1];   // m-tiles before each group

  constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
  const int n_tiles = (a.N + BN_OUT - 1) / BN_OUT;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  if (a.grp_offset) {
    for (int i = tid; i <= a.ngroups; i += 256) s_goff[i] = a.grp_offset[i];
    for (int i = tid; i < a.ngroups; i += 256) s_widx[i] = a.grp_widx ? a.grp_widx[i] : a.w_base + i;
    if (wave == 0) {   // exclusive scan of the groups' tile counts
      int before = 0;
      for (int c0 = 0; c0 < a.ngroups; c0 += 64) {
        const int g = c0 + lane;
        const int nt = g < a.ngroups ? (a.grp_offset[g + 1] - a.grp_offset[g] + BM - 1) / BM : 0;
        int incl = nt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int v = __shfl_up(incl, o, 64);
          if (lane >= o) incl += v;
        }
        if (g < a.ngroups) s_tpre[g] = before + incl - nt;
        before += __shfl(incl, 63, 64);
      }
      if (lane == 0) s_tpre[a.ngroups] = before;
    }
  }
  __syncthreads();

  // tile L of the XCD-aware order; past the end (or with nothing left) the fields of `fallback`
  // are kept, so that everything derived from a head stays addressable
  auto head_of = [&](unsigned L, const Head* fallback) {
    Head h;
    const TileMap tm = map_tile_id(L, n_tiles);
    int group;
    locate(a, s_goff, s_tpre, tm.mt, lane, group, h.m0, h.rows, h.row_base);
    h.valid = group >= 0;
    h.n0 = tm.nt * BN_OUT;
    h.widx = a.w_base;
    h.ccol = a.c_col0;
    if (h.valid) {
      h.widx = a.grp_offset ? s_widx[group] : a.w_base + group;
      h.ccol = group_col0(a, group);
    } else if (fallback) {
      h.m0 = fallback->m0; h.rows = fallback->rows; h.row_base = fallback->row_base;
      h.n0 = fallback->n0; h.widx = fallback->widx; h.ccol = fallback->ccol;
    }
    h.ccol = __builtin_amdgcn_readfirstlane(h.ccol);
    h.widx = __builtin_amdgcn_readfirstlane(h.widx);
    h.m0 = __builtin_amdgcn_readfirstlane(h.m0);
    h.rows = __builtin_amdgcn_readfirstlane(h.rows);
    h.row_base = __builtin_amdgcn_readfirstlane(h.row_base);
    h.n0 = __builtin_amdgcn_readfirstlane(h.n0);
    h.valid = __builtin_amdgcn_readfirstlane(h.valid);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = (wave * 8 + i) * 8 + (lane >> 3);
      int lr = h.m0 + r;
      if (lr >= h.rows) lr = h.rows - 1;   // rows past the group are computed and dropped
      if (lr < 0) lr = 0;
      const int logical = h.row_base + lr;
      h.raw[i] = a.a_rows ? a.a_rows[logical] : logical;
    }
    return h;
  };
  // loader role: load i (0..7) of this wave fills tile rows (wave*8 + i)*8 .. +7 of A and of B;
  // lane -> row lane/8, slot lane%8
  auto offsets_of = [&](const Head& h, aoff_t (&ao)[8], unsigned (&bo)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = (wave * 8 + i) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((r >> 1) & 7);
      ao[i] = ((aoff_t)(unsigned)h.raw[i] * (aoff_t)(unsigned)a.lda + chunk * 8) * 2;   // host: A bytes < 2^32 unless WIDE
      int ncol;
      if (SWIGLU) {
        const int half = r >> 7, q = (r & 127) >> 5, within = r & 31;
        ncol = h.n0 + half * 64 + (q >> 1) * 32 + within;   // q odd -> up matrix: loads 4..7 of every wave
      } else {
        ncol = h.n0 + r;
      }
      if (ncol >= a.N) ncol = a.N - 1;
      bo[i] = (unsigned)(((long long)ncol * a.ldb + chunk * 8) * 2);
    }
  };

  const unsigned stride = gridDim.x;   // host: tile ids + stride stay below 2^31
  unsigned L = blockIdx.x;
  Head hd = head_of(L, nullptr);
  if (!hd.valid) return;   // uniform over the block; later tiles of this block are past the end too

  const char* a_base = static_cast<const char*>(a.A);
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
  const unsigned lds_w = __builtin_amdgcn_readfirstlane(lds0 + wave * 8192);
  // fragment read offsets inside a 32-row block for the four 16-wide K steps of a tile
  int foff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    foff[kk] = (lane & 31) * 128 + (((2 * kk + (lane >> 5)) ^ ((lane >> 1) & 7)) * 16);
  const int nk = a.K / BK;   // host: >= 2

  aoff_t a_off[8];
  unsigned b_off[8];
  offsets_of(hd, a_off, b_off);
  const char* w_lo = static_cast<const char*>(a.B) + (long long)hd.widx * a.b_group_stride * 2;   // loads 0..3
  const char* w_hi = SWIGLU ? static_cast<const char*>(a.B2) + (long long)hd.widx * a.b_group_stride * 2 : w_lo;

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
  // A rows / B rows of a K tile: load g (0..7) of this wave into `stage`
  auto load_a = [&](const aoff_t (&ao)[8], int ktile, int stage, int g) {
    if constexpr (WIDE)
      load_to_lds_16(a_base + (long long)ktile * (BK * 2) + ao[g], lds_w + stage * STAGE_BYTES + g * 1024);
    else
      load_to_lds_16(a_base + (long long)ktile * (BK * 2), ao[g], lds_w + stage * STAGE_BYTES + g * 1024);
  };
  auto load_b = [&](const unsigned (&bo)[8], const char* lo, const char* hi, long long kb, int stage, int g) {
    load_to_lds_16((g < 4 ? lo : hi) + kb, bo[g], lds_w + stage * STAGE_BYTES + A_BYTES + g * 1024);
  };
  // byte offset of K tile j inside a weight row; K > kseg walks consecutive weight matrices
  // (down projection of the shared experts)
  long long kb_next = 0;
  int kin_next = 0;
  auto kb_reset = [&]() { kb_next = 0; kin_next = 0; };
  auto kb_advance = [&]() {
    kb_next += BK * 2;
    kin_next += BK;
    if (kin_next >= a.kseg) {
      kin_next = 0;
      kb_next += (a.b_group_stride - a.kseg) * 2;
    }
  };

  // prologue of the block: K tile 0 -> stage 0, its first fragments, A half of K tile 1 -> stage 1
  int par = 0;   // stage holding K tile 0 of the current output tile
#pragma unroll
  for (int g = 0; g < 8; ++g) load_a(a_off, 0, 0, g);
#pragma unroll
  for (int g = 0; g < 8; ++g) load_b(b_off, w_lo, w_hi, 0, 0, g);
  wait_all_and_barrier();
#pragma unroll
  for (int idx = 0; idx < 8; ++idx) read_frag(0, 0, 0, idx);
#pragma unroll
  for (int g = 0; g < 8; ++g) load_a(a_off, 1, 1, g);
  __builtin_amdgcn_sched_barrier(0);

  const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  __bf16* C = static_cast<__bf16*>(a.C);

  while (true) {
    // State here: K tile 0 of this output tile in stage par with its step-0 fragments in set 0;
    // the A half of K tile 1 on its way into stage par ^ 1.
    L += stride;
    const Head hn = head_of(L, &hd);   // the next tile's row gather flies during this tile's K loop
    kb_reset();
    kb_advance();

    f32x16 acc[4][4];   // [weight-row block ni][token-row block mi]
    auto mfma_pair = [&](int set, int g) {
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int t = 2 * g + q, ni = t >> 2, mi = t & 3;
        acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][ni], fa[set][mi], acc[ni][mi], 0, 0, 0);
      }
    };
    // K step 0 of the output tile: B half of K tile 1, fragments of step 1, products into zero
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      if ((g & 1) == 0) load_b(b_off, w_lo, w_hi, kb_next, par ^ 1, g >> 1);
      read_frag(1, par, 1, g);
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int t = 2 * g + q, ni = t >> 2, mi = t & 3;
        acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[0][ni], fa[0][mi], zero16, 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // steps 1 and 2 of K tile kt in stage s
    auto steps_12 = [&](int s, const unsigned (&bo)[8], const char* lo, const char* hi, long long kb) {
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        if ((g & 1) == 0) load_b(bo, lo, hi, kb, s ^ 1, 4 + (g >> 1));   // second half of the B loads begun in the step before
        read_frag(0, s, 2, g);
        mfma_pair(1, g);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        read_frag(1, s, 3, g);
        mfma_pair(0, g);
        __builtin_amdgcn_sched_barrier(0);
      }
    };

    // K tiles 0 .. nk-3: steps 1, 2, wait for K tile kt+1, step 3, step 0 of K tile kt+1
    for (int kt = 0; kt < nk - 2; ++kt) {
      const int s = (par + kt) & 1;
      steps_12(s, b_off, w_lo, w_hi, kb_next);
      kb_advance();
      // K tile kt+1 has landed (this wave's loads, then every wave's), and every wave has issued
      // and completed its last reads of stage s, which may therefore be refilled
      wait_all_and_barrier();
#pragma unroll
      for (int g = 0; g < 8; ++g) {   // step 3: A half of K tile kt+2 -> stage s, step-0 fragments of kt+1
        load_a(a_off, kt + 2, s, g);
        read_frag(0, s ^ 1, 0, g);
        mfma_pair(1, g);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int g = 0; g < 8; ++g) {   // step 0 of K tile kt+1: B half of K tile kt+2 -> stage s
        if ((g & 1) == 0) load_b(b_off, w_lo, w_hi, kb_next, s, g >> 1);
        read_frag(1, s ^ 1, 1, g);
        mfma_pair(0, g);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // K tile nk-2: as above, but the stage it frees receives K tile 0 of the next output tile
    const int s = (par + nk - 2) & 1, s1 = s ^ 1;
    steps_12(s, b_off, w_lo, w_hi, kb_next);
    wait_all_and_barrier();
    aoff_t na_off[8];
    unsigned nb_off[8];
    offsets_of(hn, na_off, nb_off);   // the gather has long landed: nothing is outstanding here
    const char* nw_lo = static_cast<const char*>(a.B) + (long long)hn.widx * a.b_group_stride * 2;
    const char* nw_hi = SWIGLU ? static_cast<const char*>(a.B2) + (long long)hn.widx * a.b_group_stride * 2 : nw_lo;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      load_a(na_off, 0, s, g);
      read_frag(0, s1, 0, g);
      mfma_pair(1, g);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      if ((g & 1) == 0) load_b(nb_off, nw_lo, nw_hi, 0, s, g >> 1);
      read_frag(1, s1, 1, g);
      mfma_pair(0, g);
      __builtin_amdgcn_sched_barrier(0);
    }
    // K tile nk-1 (stage s1): steps 1, 2; then the next tile's K tile 0 is complete in stage s and
    // stage s1 is free: step 3 sends the A half of the next tile's K tile 1 there and reads the
    // next tile's first fragments
    steps_12(s1, nb_off, nw_lo, nw_hi, 0);
    wait_all_and_barrier();
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      load_a(na_off, 1, s1, g);
      read_frag(0, s, 0, g);
      mfma_pair(1, g);
      __builtin_amdgcn_sched_barrier(0);
    }

    // epilogue.  acc[ni][mi] element r of lane l: output row (token) mi*32 + l%32, output column
    // ni*32 + (r/4)*8 + (l/32)*4 + r%4 of the wave tile: 4 consecutive columns per register quad.
    // Chunk c = 32 rows x 64 output columns = 4 KiB (128-byte rows, 16-byte slots swizzled like
    // the operand tiles), two buffers inside this wave's 8 KiB of stage s1's B region.
    {
      char* stg = smem + s1 * STAGE_BYTES + A_BYTES + wave * 8192;
      constexpr int NCH = SWIGLU ? 4 : 8;
      constexpr int W_COLS = SWIGLU ? 64 : 128;   // output columns of a wave tile
      const int srow = lane & 31;
      char* wr = stg + srow * 128 + (lane >> 5) * 8;
      const int wsw = (srow >> 1) & 7;
      const int rrow = lane >> 3, rch = lane & 7;
      // A chunk sequence number cc alternates the two staging buffers (cc & 1).  Without SAVE chunk cc is
      // output chunk cc.  With SAVE the sequence is, per row block mi: the activated chunk, then the gate
      // and the up pre-activations of the same rows (kind 0, 1, 2), so that a row block's accumulators are
      // dead after its three chunks (keeping all of them live through a second pass spills registers, and
      // every reload of a spilled register waits for the next tile's loads as well).
      auto stage = [&](int cc) {
        char* buf = wr + (cc & 1) * 4096;
        const int kind = SAVE ? cc % 3 : 0;
        const int c = SAVE ? cc / 3 : cc;
        const int mi = SWIGLU ? c : (c >> 1), h = SWIGLU ? 0 : (c & 1);
#pragma unroll
        for (int nn = 0; nn < 2; ++nn)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if (SWIGLU && kind == 0)
                v[e] = swiglu_fast(acc[2 * nn][mi][q * 4 + e], acc[2 * nn + 1][mi][q * 4 + e]);
              else if (SWIGLU)
                v[e] = acc[2 * nn + (kind - 1)][mi][q * 4 + e];   // kind 1: gate, 2: up
              else
                v[e] = acc[2 * h + nn][mi][q * 4 + e];
            }
            uint2 pk;
            pk.x = pack_bf16(v[0], v[1]);
            pk.y = pack_bf16(v[2], v[3]);
            *reinterpret_cast<uint2*>(buf + (((nn * 4 + q) ^ wsw) * 16)) = pk;
          }
      };
      // Stores go through a buffer descriptor over the wave tile's valid rows, so rows past the
      // group's end (and columns past N) are dropped by the hardware's range check: no branches.
      const int rows_left = min(hd.rows - hd.m0 - wm * 128, 128);
      const int col_w = hd.n0 + wn * W_COLS;   // first output column of the wave tile
      // (the last valid row counts only the wave tile's columns below N: with N < W_COLS and ldc = N a
      // whole tile width would reach into the next group's first row)
      // With the fused activation a wave tile is 64 columns and N a multiple of 64 (host), so a wave tile is whole
      // or wholly past N (every store of it redirected below): the constant keeps a scalar register free there.
      const int cols_left = SWIGLU ? W_COLS : min(a.N - col_w, W_COLS);
      const unsigned n_rec =
          rows_left > 0 && cols_left > 0 ? (unsigned)((rows_left - 1) * a.ldc + cols_left) * 2u : 0u;
      const unsigned long long c_tile = reinterpret_cast<unsigned long long>(
          C + (long long)(hd.row_base + hd.m0 + wm * 128) * a.ldc + hd.ccol + col_w);
      const unsigned long long c_tile_u =   // the descriptor has to sit in scalar registers
          ((unsigned long long)__builtin_amdgcn_readfirstlane((unsigned)(c_tile >> 32)) << 32) |
          (unsigned)__builtin_amdgcn_readfirstlane((unsigned)c_tile);
      const __amdgpu_buffer_rsrc_t c_rsrc = __builtin_amdgcn_make_buffer_rsrc(
          reinterpret_cast<void*>(c_tile_u), 0, __builtin_amdgcn_readfirstlane((int)n_rec), 0x00020000);
      // SAVE: the pre-activations go to rows of 2 * ldc elements, [gate | up] with the up half N columns
      // further.  One descriptor spans both halves of the wave tile's valid rows; an invalid row lies past
      // it because a row of that output is longer than N + 64 columns (2 * ldc >= 2 * N, N >= 64).
      const int ldc2 = 2 * a.ldc;
      const unsigned n_rec2 =
          SAVE && rows_left > 0 && cols_left > 0 ? (unsigned)((rows_left - 1) * ldc2 + a.N + cols_left) * 2u : 0u;
      const unsigned long long c2_tile = reinterpret_cast<unsigned long long>(
          static_cast<__bf16*>(SAVE ? a.C2 : a.C) + (long long)(hd.row_base + hd.m0 + wm * 128) * ldc2 + 2 * hd.ccol + col_w);
      const unsigned long long c2_tile_u =
          ((unsigned long long)__builtin_amdgcn_readfirstlane((unsigned)(c2_tile >> 32)) << 32) |
          (unsigned)__builtin_amdgcn_readfirstlane((unsigned)c2_tile);
      const __amdgpu_buffer_rsrc_t c2_rsrc = __builtin_amdgcn_make_buffer_rsrc(
          reinterpret_cast<void*>(c2_tile_u), 0, __builtin_amdgcn_readfirstlane((int)n_rec2), 0x00020000);
      u32x4 sv[4];
      auto read_chunk = [&](int cc) {
        const char* buf = stg + (cc & 1) * 4096;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int rl = it * 8 + rrow;   // row inside the 32-row chunk
          sv[it] = *reinterpret_cast<const u32x4*>(buf + rl * 128 + ((rch ^ ((rl >> 1) & 7)) * 16));
        }
      };
      auto store = [&](int cc) {
        const int kind = SAVE ? cc % 3 : 0;
        const int c = SAVE ? cc / 3 : cc;
        const int mi = SWIGLU ? c : (c >> 1), h = SWIGLU ? 0 : (c & 1);
        const int col = h * 64 + rch * 8;   // inside the wave tile
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int row = mi * 32 + it * 8 + rrow;
          if (kind == 0) {
            const unsigned off = col_w + col < a.N ? (unsigned)(row * a.ldc + col) * 2u : n_rec;
            __builtin_amdgcn_raw_buffer_store_b128(sv[it], c_rsrc, (int)off, 0, 0);
          } else {
            const unsigned off =
                col_w + col < a.N ? (unsigned)(row * ldc2 + col + (kind - 1) * a.N) * 2u : n_rec2;
            __builtin_amdgcn_raw_buffer_store_b128(sv[it], c2_rsrc, (int)off, 0, 0);
          }
        }
      };
      // chunk cc is converted and staged while the LDS reads of chunk cc-1 are in flight
      constexpr int NSEQ = SAVE ? 3 * NCH : NCH;
      stage(0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int cc = 1; cc < NSEQ; ++cc) {
        read_chunk(cc - 1);
        __builtin_amdgcn_sched_barrier(0);
        stage(cc);
        __builtin_amdgcn_sched_barrier(0);
        store(cc - 1);
        __builtin_amdgcn_sched_barrier(0);
      }
      read_chunk(NSEQ - 1);
      store(NSEQ - 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (!hn.valid) break;   // uniform over the block
    hd = hn;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a_off[i] = na_off[i];
      b_off[i] = nb_off[i];
    }
    w_lo = nw_lo;
    w_hi = nw_hi;
    par = s;
  }
  // the loads issued for a tile that does not exist must land before the block's LDS is released
  wait_all_and_barrier();
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
    C[(long long)(ti.row_base + row) * a.ldc + group_col0(a, ti.group) + col] = out;
  }
}

// compute units of the current device (the persistent kernel runs one block on each), cached
static int device_cu_count(int* out) {
  static int cached[64];
  int dev = 0;
  OCC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64 || cached[dev] == 0) {
    int n = 0;
    OCC_HIP(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
    OCC_REQUIRE(n > 0, OCCULT_EHIP, "device reports %d compute units", n);
    if (dev < 0 || dev >= 64) {
      *out = n;
      return OCCULT_OK;
    }
    cached[dev] = n;
  }
  *out = cached[dev];
  return OCCULT_OK;
}

// sums the K slices of a split product in slice order and rounds once: out[row][col0 + col]
__global__ __launch_bounds__(256) void splitk_reduce_bf16(const float* __restrict__ ws, int ksplit, int M, int N,
                                                          __bf16* __restrict__ out, int ldc, int col0) {
  const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;   // 4 columns per thread (N % 4 == 0)
  if (i >= (size_t)M * N) return;
  f32x4 sum = *reinterpret_cast<const f32x4*>(ws + i);
  for (int ks = 1; ks < ksplit; ++ks) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(ws + (size_t)ks * M * N + i);
    sum = sum + v;
  }
  const size_t row = i / N, col = i % N;
  uint2 pk;
  pk.x = pack_bf16(sum.x, sum.y);
  pk.y = pack_bf16(sum.z, sum.w);
  *reinterpret_cast<uint2*>(out + row * ldc + col0 + col) = pk;
}

// K slices for a product whose tiles alone would leave most of the chip idle (0 = do not split)
static int choose_ksplit(long long tiles, int nk) {
  if (tiles >= 384 || nk < 8) return 0;   // beyond that the 256-row tiles fill the chip by themselves
  long long ks = 1024 / tiles;   // about two rounds of 512 resident workgroups
  if (ks > nk / 4) ks = nk / 4;
  if (ks > 8) ks = 8;
  return ks >= 2 ? (int)ks : 0;
}

// Weights in the weight-streaming kernel's own order (bf16).  Region 1, gate and up, per weight
// matrix pair 4*f*d bytes: unit = 32 output columns, stage = 64 K elements; a stage is 8 blocks of
// 1 KiB in the order (K step ks, matrix m: gate or up, column block nb), block = 64 lanes x 16 bytes,
// lane l holding row nb*16 + l%16 of the unit at K offset ks*32 + (l/16)*8.  Region 2, down, per
// matrix 2*d*f bytes: the same with one matrix (4 blocks per stage).  One thread per 16-byte piece.
__global__ __launch_bounds__(256) void pack_weights_kernel(const u32x4* __restrict__ gate, const u32x4* __restrict__ up,
                                                           const u32x4* __restrict__ down, u32x4* __restrict__ out,
                                                           int n_mats, int d, int f) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long per1 = (long long)f * d / 4, per2 = (long long)d * f / 8;   // pieces per matrix pair / matrix
  const long long n1 = n_mats * per1;
  if (idx < n1) {
    const int e = (int)(idx / per1);
    long long rem = idx - e * per1;
    const int cb = (int)(rem / (8ll * d));           // unit: 32 columns x 2 matrices x d elements
    rem -= cb * 8ll * d;
    const int stage = (int)(rem / 512), blk = (int)(rem % 512) / 64, lane = (int)(rem % 64);
    const int ks = blk >> 2, m = (blk >> 1) & 1, nb = blk & 1;
    const int n = cb * 32 + nb * 16 + (lane & 15), k = stage * 64 + ks * 32 + (lane >> 4) * 8;
    out[idx] = (m ? up : gate)[(((long long)e * f + n) * d + k) / 8];
  } else if (idx < n1 + n_mats * per2) {
    const long long i2 = idx - n1;
    const int e = (int)(i2 / per2);
    long long rem = i2 - e * per2;
    const int cb = (int)(rem / (4ll * f));           // unit: 32 columns x f elements
    rem -= cb * 4ll * f;
    const int stage = (int)(rem / 256), blk = (int)(rem % 256) / 64, lane = (int)(rem % 64);
    const int ks = blk >> 1, nb = blk & 1;
    const int n = cb * 32 + nb * 16 + (lane & 15), k = stage * 64 + ks * 32 + (lane >> 4) * 8;
    out[idx] = down[(((long long)e * d + n) * f + k) / 8];
  }
}

// groups averaging under 24 rows take the weight-streaming kernel (one wave per 32 columns x 32 tokens)
static bool streams_weights(const GemmArgs& a, int total_rows) {
  // (that kernel addresses A rows with 32-bit byte offsets)
  return (long long)total_rows < 24ll * a.ngroups && a.N % skinny::BN_OUT == 0 &&
         (long long)a.a_rows_total * a.lda * 2 < (1ll << 32);
}

// The weight-streaming kernel over `a` (grouped rows, total_rows of them) and, when b is not NULL, over `b` in the
// same launch (uniform groups of b->M rows; same N, K and weight order as `a`, one weight matrix along K in both).
static int launch_skinny(const GemmArgs& a, const GemmArgs* b, bool swiglu, int total_rows, hipStream_t s) {
  const bool ksplit = swiglu;   // the gate/up product's waves split K; the down projection's keep whole columns
  const long long n_cb = a.N / skinny::BN_OUT;
  const long long wgs_per_mt = ksplit ? n_cb : (n_cb + 3) / 4;
  const long long a_blocks = ((total_rows + 31) / 32 + a.ngroups) * wgs_per_mt;
  long long blocks = a_blocks;
  if (b != nullptr) {
    OCC_REQUIRE(b->N == a.N && b->grp_offset == nullptr && (b->Bp != nullptr) == (a.Bp != nullptr) && a.kseg == a.K &&
                    b->K % b->kseg == 0,
                OCCULT_EINVAL, "the two problems of one weight-streaming launch differ in shape class");
    blocks += (b->ngroups * n_cb + 7) / 8 * 8 * (long long)((b->M + 31) / 32);   // whole sets of 8 units
  }
  OCC_REQUIRE(blocks < (1ll << 31), OCCULT_EINVAL, "grouped GEMM grid too large");
  const dim3 grid((unsigned)blocks), block(256);
  // the packed order holds whole matrices: a K that walks several of them steps from one matrix's stream to the next
  const bool packed = a.Bp != nullptr && (a.kseg == a.K || a.K % a.kseg == 0);
  const GemmArgs& b2 = b ? *b : a;
  const int ab = (int)a_blocks;
  if (swiglu && packed) hipLaunchKernelGGL((skinny::grouped_gemm_bf16<true, 2, true, true>), grid, block, 0, s, a, b2, ab);
  else if (swiglu) hipLaunchKernelGGL((skinny::grouped_gemm_bf16<true, 2, false, true>), grid, block, 0, s, a, b2, ab);
  else if (packed) hipLaunchKernelGGL((skinny::grouped_gemm_bf16<false, 2, true, false>), grid, block, 0, s, a, b2, ab);
  else hipLaunchKernelGGL((skinny::grouped_gemm_bf16<false, 2, false, false>), grid, block, 0, s, a, b2, ab);
  OCC_LAUNCH_CHECK("grouped_gemm");
  return OCCULT_OK;
}

// *fused_save: the pre-activations asked for through a.C2 were written by the launch itself
static int launch_gemm_main(const occult_cfg_t& c, const GemmArgs& a, bool swiglu, int total_rows, hipStream_t s,
                            bool* fused_save_out) {
  *fused_save_out = false;
  if (c.dtype == OCCULT_BF16) {
    const int groups = a.ngroups;
    // 256-row tiles once groups average enough rows and there are at least two K tiles to pipeline
    // (an A operand of 4 GiB or more takes the variant with 64-bit row offsets)
    // (measured on 60 experts, d = 2048, f = 1408: the gate/up product is weight-bound on the
    // 128-row tiles until an expert's rows no longer fit one of them; the down projection is
    // faster on the 256-row tiles from about 64 rows per expert)
    const long long big_rows = a.grp_offset == nullptr ? 192 : (swiglu ? 129 : 64);
    const bool use_big =
        (long long)total_rows >= big_rows * groups && a.ksplit <= 1 && a.K >= 2 * t256::BK && a.N % 64 == 0;
    const bool wide = (long long)a.a_rows_total * a.lda * 2 >= (1ll << 32);
    // only the 256-row tiles store the pre-activations themselves (not built with 64-bit offsets: registers)
    const bool fused_save = swiglu && a.C2 != nullptr && use_big && !wide;
    *fused_save_out = fused_save;
    const bool use_skinny = !use_big && streams_weights(a, total_rows);
    if (use_skinny) return launch_skinny(a, nullptr, swiglu, total_rows, s);
    const int bm = use_big ? t256::BM : small::BM;
    const int bn = use_big ? t256::BN : small::BN;
    const int bn_out = swiglu ? bn / 2 : bn;
    const long long m_tiles = (total_rows + bm - 1) / bm + a.ngroups;
    long long blocks = mapped_grid(m_tiles, (a.N + bn_out - 1) / bn_out);
    OCC_REQUIRE(blocks < (1ll << 31), OCCULT_EINVAL, "grouped GEMM grid too large");
    if (use_big) {   // persistent: one block per CU, a multiple of 8 so a block keeps its XCD
      int cus = 0;
      const int rc = device_cu_count(&cus);
      if (rc) return rc;
      const long long resident = cus >= 8 ? cus / 8 * 8 : 8;
      if (blocks > resident) blocks = resident;
    }
    const bool split = !use_big && !swiglu && a.ksplit > 1;   // caller set ksplit and ws (one group)
    GemmArgs b = a;
    if (!split) b.ksplit = 0;
    // the XCD-aware order pads the grid to whole chunks per XCD: pointless when there are few tiles
    const long long plain_blocks = m_tiles * ((a.N + bn_out - 1) / bn_out);
    if (!use_big && plain_blocks <= 512) {
      b.plain_map = 1;
      blocks = plain_blocks;
    }
    const dim3 grid((unsigned)blocks, split ? (unsigned)b.ksplit : 1u), block(256);
    if (use_big) {
      if (swiglu && fused_save) hipLaunchKernelGGL((t256::grouped_gemm_bf16<true, true>), grid, block, 0, s, b);
      else if (swiglu && wide) hipLaunchKernelGGL((t256::grouped_gemm_bf16<true, false, true>), grid, block, 0, s, b);
      else if (swiglu) hipLaunchKernelGGL((t256::grouped_gemm_bf16<true, false>), grid, block, 0, s, b);
      else if (wide) hipLaunchKernelGGL((t256::grouped_gemm_bf16<false, false, true>), grid, block, 0, s, b);
      else hipLaunchKernelGGL((t256::grouped_gemm_bf16<false, false>), grid, block, 0, s, b);
    } else {
      if (swiglu) hipLaunchKernelGGL(small::grouped_gemm_bf16<true>, grid, block, 0, s, b);
      else hipLaunchKernelGGL(small::grouped_gemm_bf16<false>, grid, block, 0, s, b);
    }
    if (split) {
      OCC_LAUNCH_CHECK("grouped_gemm");
      const size_t quads = (size_t)b.M * b.N / 4;
      hipLaunchKernelGGL(splitk_reduce_bf16, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, b.ws, b.ksplit,
                         b.M, b.N, static_cast<__bf16*>(b.C), b.ldc, b.c_col0);
    }
  } else {
    const long long m_tiles = (total_rows + FM - 1) / FM + a.ngroups;
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

// The two pre-activations of a gate/up product `a` (a.C2) as two more products without the activation: only the
// 256-row tiles store them from the product's own launch.
static int launch_preactivations(const occult_cfg_t& c, const GemmArgs& a, int total_rows, hipStream_t s) {
  bool fused_save = false;
  GemmArgs p = a;
  p.C = a.C2; p.ldc = 2 * a.ldc; p.c_group_cols = 2 * a.c_group_cols; p.C2 = nullptr; p.B2 = nullptr; p.Bp = nullptr;
  p.c_col0 = 2 * a.c_col0;
  int rc = launch_gemm_main(c, p, false, total_rows, s, &fused_save);
  if (rc) return rc;
  p.B = a.B2; p.c_col0 = 2 * a.c_col0 + a.N;
  return launch_gemm_main(c, p, false, total_rows, s, &fused_save);
}

int launch_gemm(const occult_cfg_t& c, const GemmArgs& a, bool swiglu, int total_rows, hipStream_t s) {
  if (total_rows == 0) return OCCULT_OK;
  bool fused_save = false;
  int rc = launch_gemm_main(c, a, swiglu, total_rows, s, &fused_save);
  if (rc) return rc;
  if (swiglu && a.C2 != nullptr && !fused_save) rc = launch_preactivations(c, a, total_rows, s);
  return rc;
}

}  // namespace occult

using namespace occult;


// Scratch that lets the shared experts' down projection of a small batch be split over K: the
// product has T/128 x d/128 tiles only (16 for T = 128, d = 2048) with a long K = S*f.
// Small batches whose routed experts take the weight-streaming kernel: the shared experts ride in the same two
// launches, the down projection as one product whose K walks the S matrices (no scratch, no extra launch).
constexpr int kPairMaxT = 128;   // a shared expert's weights are requested once per 32 tokens (from L2 after the first)
static bool pairs_shared_with_routed(const occult_cfg_t& c) {
  return c.dtype == OCCULT_BF16 && c.S > 0 && c.T > 0 && c.T <= kPairMaxT && (long long)c.T * c.k < 24ll * c.E &&
         c.f % skinny::BN_OUT == 0 && c.d % skinny::BN_OUT == 0 &&
         (long long)sfd_rows_max(c) * c.d * 2 < (1ll << 32) && (long long)c.T * c.k * c.f * 2 < (1ll << 32) &&
         (long long)c.T * c.S * c.f * 2 < (1ll << 32);
}

static size_t ffn_ws_need(const occult_cfg_t& c, int* ksplit_out) {
  *ksplit_out = 0;
  if (c.S == 0 || c.dtype != OCCULT_BF16 || c.T == 0) return 0;
  if (c.T < 24) return 0;   // those batches take the weight-streaming kernel
  if (pairs_shared_with_routed(c)) return 0;   // the shared experts run inside the routed experts' launches
  const long long tiles = (long long)((c.T + 127) / 128) * ((c.d + 127) / 128);
  const int ks = choose_ksplit(tiles, c.S * c.f / 64);
  if (ks == 0 || c.d % 4 != 0) return 0;
  *ksplit_out = ks;
  return (size_t)ks * c.T * c.d * sizeof(float);
}

extern "C" int occult_expert_ffn_ws_bytes(const occult_cfg_t* cfg, size_t* ws_bytes) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  OCC_REQUIRE(ws_bytes, OCCULT_ENULLPTR, "ws_bytes is NULL");
  int ks = 0;
  *ws_bytes = ffn_ws_need(*cfg, &ks);
  return OCCULT_OK;
}

static int expert_ffn_impl(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                           const void* x, const occult_weights_t* weights, const void* packed, void* epd_h,
                           void* epd_y, void* h_shared, void* y_shared, void* ws, size_t ws_bytes,
                           occult_stream_t stream, void* epd_gu = nullptr, void* gu_shared = nullptr) {
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

  hipStream_t s_shared = s;
  const bool do1 = c.ffn_phase != 2, do2 = c.ffn_phase != 1;

  auto shared_experts = [&]() -> int {
    // h_shared[t][s*f .. (s+1)*f) per shared expert, then one product whose K dimension walks
    // the S down-projection matrices
    if (do1) {   // the S shared experts as S groups over the same T rows
      GemmArgs a1{};
      a1.A = x; a1.lda = c.d; a1.a_rows = nullptr;
      a1.B = weights->w_gate; a1.B2 = weights->w_up;
      a1.b_group_stride = (long long)c.f * c.d; a1.ldb = c.d; a1.kseg = c.d;
      a1.C = h_shared; a1.ldc = c.S * c.f; a1.c_col0 = 0; a1.c_group_cols = c.f;
      a1.C2 = gu_shared;   // rows of S * 2f: per shared expert [gate | up]
      a1.grp_offset = nullptr; a1.grp_widx = nullptr; a1.w_base = c.E;
      a1.ngroups = c.S; a1.M = c.T; a1.N = c.f; a1.K = c.d; a1.a_rows_total = c.T;
      const int r1 = launch_gemm(c, a1, true, c.T * c.S, s_shared);
      if (r1) return r1;
    }
    if (do2) {
      GemmArgs a2{};
      a2.A = h_shared; a2.lda = c.S * c.f; a2.a_rows = nullptr;
      a2.B = weights->w_down; a2.B2 = nullptr;
      a2.b_group_stride = (long long)c.d * c.f; a2.ldb = c.f; a2.kseg = c.f;
      a2.C = y_shared; a2.ldc = c.d; a2.c_col0 = 0;
      a2.grp_offset = nullptr; a2.grp_widx = nullptr; a2.w_base = c.E;
      a2.ngroups = 1; a2.M = c.T; a2.N = c.d; a2.K = c.S * c.f; a2.a_rows_total = c.T;
      int ks = 0;
      const size_t need = ffn_ws_need(c, &ks);
      if (ks > 1 && ws != nullptr && ws_bytes >= need) {
        a2.ksplit = ks;
        a2.ws = static_cast<float*>(ws);
      }
      return launch_gemm(c, a2, false, c.T, s_shared);
    }
    return OCCULT_OK;
  };
  auto routed_experts = [&]() -> int {
    if (do1) {
      GemmArgs g1{};
      g1.A = sfd_x; g1.lda = c.d; g1.a_rows = plan->epd_sfd_row;
      g1.B = weights->w_gate; g1.B2 = weights->w_up;
      g1.b_group_stride = (long long)c.f * c.d; g1.ldb = c.d; g1.kseg = c.d;
      g1.Bp = packed; g1.bp_group_stride = 4ll * c.f * c.d;
      g1.C = epd_h; g1.ldc = c.f; g1.c_col0 = 0;
      g1.C2 = epd_gu;      // rows of 2f: [gate | up]
      g1.grp_offset = plan->exp_offset; g1.grp_widx = plan->pos_expert; g1.w_base = 0;
      g1.ngroups = c.E; g1.M = 0; g1.N = c.f; g1.K = c.d;
      g1.a_rows_total = sfd_rows_max(c);
      const int r1 = launch_gemm(c, g1, true, n_epd, s);
      if (r1) return r1;
    }
    if (do2) {
      GemmArgs g2{};
      g2.A = epd_h; g2.lda = c.f; g2.a_rows = nullptr;
      g2.B = weights->w_down; g2.B2 = nullptr;
      g2.b_group_stride = (long long)c.d * c.f; g2.ldb = c.f; g2.kseg = c.f;
      if (packed) g2.Bp = static_cast<const char*>(packed) + 4ll * c.f * c.d * (c.E + c.S);
      g2.bp_group_stride = 2ll * c.d * c.f;
      g2.C = epd_y; g2.ldc = c.d; g2.c_col0 = 0;
      g2.grp_offset = plan->exp_offset; g2.grp_widx = plan->pos_expert; g2.w_base = 0;
      g2.ngroups = c.E; g2.M = 0; g2.N = c.d; g2.K = c.f;
      g2.a_rows_total = n_epd;
      return launch_gemm(c, g2, false, n_epd, s);
    }
    return OCCULT_OK;
  };

  if (pairs_shared_with_routed(c)) {
    if (do1) {
      GemmArgs g1{}, a1{};
      g1.A = sfd_x; g1.lda = c.d; g1.a_rows = plan->epd_sfd_row;
      a1.A = x; a1.lda = c.d;
      g1.B = a1.B = weights->w_gate; g1.B2 = a1.B2 = weights->w_up;
      g1.b_group_stride = a1.b_group_stride = (long long)c.f * c.d;
      g1.ldb = a1.ldb = g1.kseg = a1.kseg = g1.K = a1.K = c.d;
      g1.Bp = a1.Bp = packed; g1.bp_group_stride = a1.bp_group_stride = 4ll * c.f * c.d;
      g1.N = a1.N = c.f;
      g1.C = epd_h; g1.ldc = c.f;
      a1.C = h_shared; a1.ldc = c.S * c.f; a1.c_group_cols = c.f;
      g1.grp_offset = plan->exp_offset; g1.grp_widx = plan->pos_expert; g1.ngroups = c.E;
      g1.a_rows_total = sfd_rows_max(c);
      a1.w_base = c.E; a1.ngroups = c.S; a1.M = c.T; a1.a_rows_total = c.T;
      rc = launch_skinny(g1, &a1, true, n_epd, s);
      if (rc) return rc;
      if (epd_gu != nullptr) {   // a training step keeps the pre-activations: rows of 2f, [gate | up]
        g1.C2 = epd_gu;
        rc = launch_preactivations(c, g1, n_epd, s);
        if (rc) return rc;
      }
      if (gu_shared != nullptr) {   // rows of S * 2f: per shared expert [gate | up]
        a1.C2 = gu_shared;
        rc = launch_preactivations(c, a1, c.T * c.S, s);
        if (rc) return rc;
      }
    }
    if (do2) {
      GemmArgs g2{}, a2{};
      g2.A = epd_h; g2.lda = c.f;
      a2.A = h_shared; a2.lda = c.S * c.f;
      g2.B = a2.B = weights->w_down;
      g2.b_group_stride = a2.b_group_stride = (long long)c.d * c.f;
      g2.ldb = a2.ldb = g2.kseg = a2.kseg = g2.K = c.f;
      a2.K = c.S * c.f;   // one product over the S down matrices
      if (packed) g2.Bp = a2.Bp = static_cast<const char*>(packed) + 4ll * c.f * c.d * (c.E + c.S);
      g2.bp_group_stride = a2.bp_group_stride = 2ll * c.d * c.f;
      g2.N = a2.N = c.d;
      g2.C = epd_y; g2.ldc = c.d;
      a2.C = y_shared; a2.ldc = c.d;
      g2.grp_offset = plan->exp_offset; g2.grp_widx = plan->pos_expert; g2.ngroups = c.E;
      g2.a_rows_total = n_epd;
      a2.w_base = c.E; a2.ngroups = 1; a2.M = c.T; a2.a_rows_total = c.T;
      rc = launch_skinny(g2, &a2, false, n_epd, s);
      if (rc) return rc;
    }
    return OCCULT_OK;
  }
  rc = routed_experts();
  if (rc) return rc;
  if (c.S > 0) {
    rc = shared_experts();
    if (rc) return rc;
  }
  return OCCULT_OK;
}

extern "C" int occult_expert_ffn(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                 const void* x, const occult_weights_t* weights, void* epd_h, void* epd_y,
                                 void* h_shared, void* y_shared, occult_stream_t stream) {
  return expert_ffn_impl(cfg, plan, sfd_x, x, weights, nullptr, epd_h, epd_y, h_shared, y_shared, nullptr, 0, stream);
}

extern "C" int occult_expert_ffn_ws(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                    const void* x, const occult_weights_t* weights, void* epd_h, void* epd_y,
                                    void* h_shared, void* y_shared, void* ws, size_t ws_bytes,
                                    occult_stream_t stream) {
  if (ws != nullptr) OCC_REQUIRE(aligned16(ws), OCCULT_EALIGN, "ws is not 16-byte aligned");
  return expert_ffn_impl(cfg, plan, sfd_x, x, weights, nullptr, epd_h, epd_y, h_shared, y_shared, ws, ws_bytes, stream);
}

extern "C" int occult_expert_ffn_train(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                       const void* x, const occult_weights_t* weights, void* epd_h, void* epd_y,
                                       void* h_shared, void* y_shared, void* epd_gu, void* gu_shared, void* ws,
                                       size_t ws_bytes, occult_stream_t stream) {
  OCC_REQUIRE(epd_gu != nullptr, OCCULT_ENULLPTR, "epd_gu is NULL");
  OCC_REQUIRE(cfg == nullptr || cfg->S == 0 || gu_shared != nullptr, OCCULT_ENULLPTR, "gu_shared is NULL with shared experts");
  OCC_REQUIRE(aligned16(epd_gu) && aligned16(gu_shared) && aligned16(ws), OCCULT_EALIGN, "a buffer is not 16-byte aligned");
  return expert_ffn_impl(cfg, plan, sfd_x, x, weights, nullptr, epd_h, epd_y, h_shared, y_shared, ws, ws_bytes, stream,
                         epd_gu, gu_shared);
}

static size_t packed_bytes(const occult_cfg_t& c) {
  return c.dtype == OCCULT_BF16 ? (size_t)(c.E + c.S) * 3 * c.d * c.f * 2 : 0;
}

extern "C" int occult_pack_weights_bytes(const occult_cfg_t* cfg, size_t* bytes) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  OCC_REQUIRE(bytes, OCCULT_ENULLPTR, "bytes is NULL");
  *bytes = packed_bytes(*cfg);
  return OCCULT_OK;
}

extern "C" int occult_pack_weights(const occult_cfg_t* cfg, const occult_weights_t* weights, void* packed,
                                   size_t packed_size, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.dtype != OCCULT_BF16) return OCCULT_OK;   // the f32 path has no weight-streaming kernel
  OCC_REQUIRE(weights && weights->w_gate && weights->w_up && weights->w_down && packed, OCCULT_ENULLPTR,
              "weights, one of its tensors or packed is NULL");
  OCC_REQUIRE(c.d % 64 == 0 && c.f % 64 == 0, OCCULT_ESHAPE,
              "bf16 path needs d and f to be multiples of 64 (d=%d, f=%d)", c.d, c.f);
  OCC_REQUIRE(packed_size >= packed_bytes(c), OCCULT_EWORKSPACE, "packed buffer of %zu bytes < required %zu", packed_size,
              packed_bytes(c));
  OCC_REQUIRE(aligned16(weights->w_gate) && aligned16(weights->w_up) && aligned16(weights->w_down) && aligned16(packed),
              OCCULT_EALIGN, "a buffer is not 16-byte aligned");
  const long long pieces = (long long)packed_bytes(c) / 16;
  OCC_REQUIRE((pieces + 255) / 256 < (1ll << 31), OCCULT_EINVAL, "too many weights for one launch");
  hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const u32x4*>(weights->w_gate),
                     static_cast<const u32x4*>(weights->w_up), static_cast<const u32x4*>(weights->w_down),
                     static_cast<u32x4*>(packed), c.E + c.S, c.d, c.f);
  OCC_LAUNCH_CHECK("pack_weights_kernel");
  return OCCULT_OK;
}

extern "C" int occult_expert_ffn_packed(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                        const void* x, const occult_weights_t* weights, const void* packed,
                                        void* epd_h, void* epd_y, void* h_shared, void* y_shared, void* ws,
                                        size_t ws_bytes, occult_stream_t stream) {
  if (ws != nullptr) OCC_REQUIRE(aligned16(ws), OCCULT_EALIGN, "ws is not 16-byte aligned");
  if (packed != nullptr) OCC_REQUIRE(aligned16(packed), OCCULT_EALIGN, "packed is not 16-byte aligned");
  const void* use = (cfg && cfg->dtype == OCCULT_BF16) ? packed : nullptr;
  return expert_ffn_impl(cfg, plan, sfd_x, x, weights, use, epd_h, epd_y, h_shared, y_shared, ws, ws_bytes, stream);
}
