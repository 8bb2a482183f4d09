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
// bf16 kernel.  Block = 256 threads = 4 waves (2 x 2), block tile 256 x 256 outputs, wave tile
// 128 x 128 = 4 x 4 v_mfma_f32_32x32x16_bf16 tiles (256 accumulator registers, one block per CU),
// 64 rows per step.  The MFMA operands want 8 consecutive contracted elements per lane, which in
// memory are 8 different rows: a thread loads 16-byte vectors (8 columns) of 4 consecutive rows,
// transposes the 4 x 8 block in registers (v_perm_b32) and writes eight 8-byte pieces to an LDS tile
// laid out [column][64 rows], so the fragment reads are the forward kernels' 16-byte reads.  LDS
// rows are 128 bytes; 16-byte chunk c of row m sits at chunk c ^ (((m >> 1) ^ (m >> 3)) & 7), which
// spreads both access patterns over the banks: fragment reads (32 consecutive rows, two chunks)
// and transposed writes (rows 8 apart, two adjacent halves).  Two LDS stages: the global loads of
// step s+1 are in flight during the products of step s and are written to the other stage after
// them; one barrier per step.  Outputs are f32 (gradient accumulation across calls is exact to f32),
// stored straight from the accumulators: 32 lanes cover 128 contiguous bytes.
// A group's tiles are launched on one XCD (workgroup id % 8), so its rows are fetched into one L2.
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
};

namespace wg {
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int OP_BYTES = 256 * 128;   // one operand tile: 256 columns x 64 rows of bf16
constexpr int STAGE_BYTES = 2 * OP_BYTES;

__device__ __forceinline__ int swz(int m) { return ((m >> 1) ^ (m >> 3)) & 7; }

__global__ __launch_bounds__(256) void wgrad_bf16(const WgradArgs a) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int nt_n = (a.N + BN - 1) / BN;
  const int tiles = ((a.M + BM - 1) / BM) * nt_n;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int group = (slot / tiles) * 8 + xcd;
  if (group >= a.ngroups) return;   // whole block; before any barrier
  const int tile = slot % tiles;
  const int m0 = (tile / nt_n) * BM, n0 = (tile % nt_n) * BN;
  int r0 = 0, r1 = a.R;
  if (a.grp_offset) {
    r0 = a.grp_offset[group];
    r1 = a.grp_offset[group + 1];
  }
  const long long widx = a.grp_widx ? a.grp_widx[group] : (a.w_base + group);
  const int nk = (r1 - r0 + BK - 1) / BK;

  // loader role: vector column vm (8 elements), row quad rq of each 32-row half of a step
  const int vm = tid & 31, rq = tid >> 5;
  const bool a_ok = m0 + vm * 8 < a.M, b_ok = n0 + vm * 8 < a.N;   // host: M % 8 == 0, N % 8 == 0
  const char* a_base = static_cast<const char*>(a.A) + (long long)(a.a_col0 + group * a.a_group_cols + m0 + vm * 8) * 2;
  const char* b_base = static_cast<const char*>(a.B) + (long long)(a.b_col0 + group * a.b_group_cols + n0 + vm * 8) * 2;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  u32x4 ra[2][4], rb[2][4];
  auto load = [&](int s) {
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = r0 + s * BK + p * 32 + rq * 4 + i;
        const bool in = r < r1;   // rows past the group's end contribute zeros
        ra[p][i] = zero4;
        rb[p][i] = zero4;
        if (in && a_ok) ra[p][i] = *reinterpret_cast<const u32x4*>(a_base + (long long)r * a.lda * 2);
        if (in && b_ok) {
          const long long src = a.b_rows ? a.b_rows[r] : r;
          rb[p][i] = *reinterpret_cast<const u32x4*>(b_base + src * a.ldb * 2);
        }
      }
  };
  // 4 rows x 8 columns in registers -> eight (column, 4 rows) pieces of 8 bytes
  auto write_op = [&](char* dst, const u32x4 (&v)[2][4]) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int kq = p * 8 + rq;   // which group of 4 rows of the step
#pragma unroll
      for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const unsigned sel = h ? 0x07060302u : 0x05040100u;
          uint2 piece;
          piece.x = __builtin_amdgcn_perm(v[p][1][d], v[p][0][d], sel);
          piece.y = __builtin_amdgcn_perm(v[p][3][d], v[p][2][d], sel);
          const int col = vm * 8 + d * 2 + h;
          *reinterpret_cast<uint2*>(dst + col * 128 + (((kq >> 1) ^ swz(col)) * 16) + (kq & 1) * 8) = piece;
        }
    }
  };
  auto write = [&](int buf) {
    char* st = smem + buf * STAGE_BYTES;
    write_op(st, ra);
    write_op(st + OP_BYTES, rb);
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mi][ni][e] = 0.0f;

  const int frow = lane & 31, fk = lane >> 5;
  auto compute = [&](int buf) {
    const char* As = smem + buf * STAGE_BYTES;
    const char* Bs = As + OP_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[4], fb[4];
      const int c = ks * 2 + fk;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ml = wm * 128 + i * 32 + frow, nl = wn * 128 + i * 32 + frow;
        fa[i] = *reinterpret_cast<const bf16x8*>(As + ml * 128 + ((c ^ swz(ml)) * 16));
        fb[i] = *reinterpret_cast<const bf16x8*>(Bs + nl * 128 + ((c ^ swz(nl)) * 16));
      }
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
    }
  };

  if (nk > 0) {
    load(0);
    write(0);
  }
  __syncthreads();
  for (int s = 0; s < nk; ++s) {
    const bool more = s + 1 < nk;   // block-uniform
    if (more) load(s + 1);
    compute(s & 1);
    if (more) write((s + 1) & 1);
    __syncthreads();
  }

  // accumulator element e of lane l: output row (e / 4) * 8 + (l / 32) * 4 + e % 4, column l % 32 of its 32 x 32 tile
  float* cmat = a.C + widx * a.c_mat_stride;
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int n = n0 + wn * 128 + ni * 32 + frow;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * 128 + mi * 32 + (e >> 2) * 8 + fk * 4 + (e & 3);
        if (m < a.M && n < a.N) {
          float* p = cmat + (long long)m * a.ldc + n;
          float v = acc[mi][ni][e];
          if (a.accumulate) v += *p;
          *p = v;
        }
      }
    }
}
}  // namespace wg

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

static int launch_wgrad(const occult_cfg_t& c, const WgradArgs& a, hipStream_t s) {
  if (a.ngroups == 0 || a.M == 0 || a.N == 0) return OCCULT_OK;
  if (c.dtype == OCCULT_BF16) {
    const long long tiles = (long long)((a.M + wg::BM - 1) / wg::BM) * ((a.N + wg::BN - 1) / wg::BN);
    const long long blocks = (long long)((a.ngroups + 7) / 8) * tiles * 8;
    OCC_REQUIRE(blocks < (1ll << 31), OCCULT_EINVAL, "weight-gradient grid too large");
    hipLaunchKernelGGL(wg::wgrad_bf16, dim3((unsigned)blocks), dim3(256), 0, s, a);
  } else {
    OCC_REQUIRE(a.ngroups <= 65535, OCCULT_EINVAL, "too many groups");
    hipLaunchKernelGGL(wgrad_f32, dim3((a.N + 15) / 16, (a.M + 15) / 16, a.ngroups), dim3(256), 0, s, a);
  }
  OCC_LAUNCH_CHECK("wgrad");
  return OCCULT_OK;
}

}  // namespace occult

using namespace occult;

extern "C" int occult_expert_ffn_backward_weights(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                                  const void* x, const void* epd_h, const void* h_shared,
                                                  const void* epd_dy, const void* dy, const void* epd_gu,
                                                  const void* gu_shared, float* dw_gate, float* dw_up, float* dw_down,
                                                  int accumulate, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
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
      rc = launch_wgrad(c, a, s);
      if (rc) return rc;
    }
    for (int up = 0; up < 2; ++up) {   // dW_gate, dW_up [f][d] = sum_r dg_r (x) x_r, sum_r du_r (x) x_r
      WgradArgs a = base;
      a.A = sh ? gu_shared : epd_gu; a.lda = sh ? c.S * 2 * c.f : 2 * c.f; a.a_col0 = up ? c.f : 0;
      a.a_group_cols = sh ? 2 * c.f : 0; a.M = c.f;
      a.B = sh ? x : sfd_x; a.ldb = c.d; a.b_rows = sh ? nullptr : plan->epd_sfd_row; a.N = c.d;
      a.C = up ? dw_up : dw_gate; a.c_mat_stride = mat; a.ldc = c.d;
      rc = launch_wgrad(c, a, s);
      if (rc) return rc;
    }
  }
  return OCCULT_OK;
}
