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
  int N;                    // output columns (for SWIGLU: columns of h)
  int K;
};

struct TileInfo {
  int group, m0, rows, row_base;
};

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
// bf16 MFMA kernel.  Block = 256 threads = 4 waves (2 x 2), block tile 128 x 128 x 64,
// wave tile 64 x 64 = 2 x 2 MFMA tiles of 32 x 32.  With SWIGLU the 128 B-rows of a tile are
// [gate n0..n0+31 | up n0..n0+31 | gate n0+32..n0+63 | up n0+32..n0+63], so the two MFMA
// columns of a wave hold gate and up of the same 32 output columns.
constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_STRIDE = BK + 8;   // 144-byte rows: 16-byte reads of 8 consecutive rows hit 8 distinct bank groups

template <bool SWIGLU>
__global__ __launch_bounds__(256) void grouped_gemm_bf16(const GemmArgs a) {
  __shared__ __attribute__((aligned(16))) __bf16 As[BM * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) __bf16 Bs[BN * LDS_STRIDE];
  __shared__ TileInfo s_info;

  constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
  const int n_tiles = (a.N + BN_OUT - 1) / BN_OUT;
  const int mt = blockIdx.x / n_tiles;
  const int n0 = (blockIdx.x % n_tiles) * BN_OUT;
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
    const int bn_out = swiglu ? BN / 2 : BN;
    const long long m_tiles = (total_rows + BM - 1) / BM + (a.grp_offset ? a.ngroups : 0);
    const long long blocks = m_tiles * ((a.N + bn_out - 1) / bn_out);
    OCC_REQUIRE(blocks < (1ll << 31), OCCULT_EINVAL, "grouped GEMM grid too large");
    if (swiglu)
      hipLaunchKernelGGL(grouped_gemm_bf16<true>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL(grouped_gemm_bf16<false>, dim3((unsigned)blocks), dim3(256), 0, s, a);
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
    OCC_REQUIRE(c.d % BK == 0 && c.f % BK == 0, OCCULT_ESHAPE,
                "bf16 path needs d and f to be multiples of %d (d=%d, f=%d)", BK, c.d, c.f);
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
      a1.ngroups = 1; a1.M = c.T; a1.N = c.f; a1.K = c.d;
      rc = launch_gemm(c, a1, true, c.T, s);
      if (rc) return rc;
    }
    GemmArgs a2{};
    a2.A = h_shared; a2.lda = c.S * c.f; a2.a_rows = nullptr;
    a2.B = weights->w_down; a2.B2 = nullptr;
    a2.b_group_stride = (long long)c.d * c.f; a2.ldb = c.f; a2.kseg = c.f;
    a2.C = y_shared; a2.ldc = c.d; a2.c_col0 = 0;
    a2.grp_offset = nullptr; a2.grp_widx = nullptr; a2.w_base = c.E;
    a2.ngroups = 1; a2.M = c.T; a2.N = c.d; a2.K = c.S * c.f;
    if (do2) {
      rc = launch_gemm(c, a2, false, c.T, s);
      if (rc) return rc;
    }
  }
  return OCCULT_OK;
}
