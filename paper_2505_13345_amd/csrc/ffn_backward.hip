// Backward pass of the expert computation: input gradients of the grouped SwiGLU experts.
//
// The paper trains through the layer (Introduction; Sec. 4, Training) with the same sparse
// products as the forward pass and prints no backward algorithm; this is the chain rule through
// the expert of the forward pass (App. A.2 "SMM with Scattering" / "SMM with Merging"), on the
// same plan.  For EPD row q of the expert at position P, with x_q = sfd_x[epd_sfd_row[q]]:
//   g = W_gate x_q, u = W_up x_q                      recomputed (the forward keeps only silu(g) * u)
//   dh = W_down^T epd_dy[q]
//   dg = dh * u * silu'(g),  du = dh * silu(g)         silu'(g) = s (1 + g (1 - s)), s = 1 / (1 + e^-g)
//   epd_dx[q] = W_gate^T dg + W_up^T du
// All four products are the forward's grouped GEMM (gemm.h) with other operands: the two products
// that contract over the weights' row index read transposed copies of the weights, written once
// per weight update by occult_transpose_weights ([f][d] down projection; [d][2f] gate | up side by
// side, so that the last product is one GEMM over K = 2f).  Shared experts: the same four products
// over all T rows, the shared weights as uniform groups.
#include "common.h"
#include "gemm.h"

namespace occult {

// out[m][c][col0 + r] = in[m][r][c] for matrices of R x C elements; 64 x 64 tiles through LDS
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, T* __restrict__ out, int R, int C,
                                                        long long out_mat_stride, int out_ld, int col0) {
  __shared__ T tile[64][65];
  const int m = blockIdx.z;
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const T* src = in + (size_t)m * R * C;
  T* dst = out + (size_t)m * out_mat_stride;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    if (r < R && c < C) tile[i][tx] = src[(size_t)r * C + c];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (r < R && c < C) dst[(size_t)c * out_ld + col0 + r] = tile[tx][i];
  }
}

// The same for 2-byte elements with 16-byte global accesses on both sides (R % 8 == 0, C % 8 == 0):
// a thread loads 8 columns of two rows, scatters them into the LDS tile as [column][row], and reads
// back 8 consecutive rows of one column as one vector.  LDS rows are padded to 72 elements (144
// bytes), which keeps the vectors 16-byte aligned.
__global__ __launch_bounds__(256) void transpose16_kernel(const unsigned short* __restrict__ in,
                                                          unsigned short* __restrict__ out, int R, int C,
                                                          long long out_mat_stride, int out_ld, int col0) {
  __shared__ __attribute__((aligned(16))) unsigned short tile[64][72];
  const int m = blockIdx.z;
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const unsigned short* src = in + (size_t)m * R * C;
  unsigned short* dst = out + (size_t)m * out_mat_stride;
  const int v = threadIdx.x & 7, q = threadIdx.x >> 3;   // vector of 8 inside 64, row (or column) 0..31
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int r = r0 + q + 32 * h, c = c0 + v * 8;
    if (r < R && c < C) {
      const u32x4 x = *reinterpret_cast<const u32x4*>(src + (size_t)r * C + c);
      const unsigned w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        tile[v * 8 + 2 * j][q + 32 * h] = (unsigned short)(w[j] & 0xFFFFu);
        tile[v * 8 + 2 * j + 1][q + 32 * h] = (unsigned short)(w[j] >> 16);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int c = c0 + q + 32 * h, r = r0 + v * 8;
    if (r < R && c < C)
      *reinterpret_cast<u32x4*>(dst + (size_t)c * out_ld + col0 + r) = *reinterpret_cast<const u32x4*>(&tile[q + 32 * h][v * 8]);
  }
}

// gu[row] = [g | u] (2f elements), dh[row] (f elements)  ->  gu[row] = [dg | du], in place.
// One thread per 16-byte vector of a row of f elements.
template <bool BF16>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(void* __restrict__ gu, const void* __restrict__ dh,
                                                         long long rows, int f) {
  using R = Row<BF16>;
  constexpr int NE = R::kElems;
  const int vecs = f / NE;   // host: f * element size is a multiple of 16
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * vecs) return;
  const long long row = i / vecs;
  const int c = (int)(i - row * vecs);
  float g[NE], u[NE], h[NE];
  R::load(gu, (size_t)row, 2 * vecs, c, g);
  R::load(gu, (size_t)row, 2 * vecs, vecs + c, u);
  R::load(dh, (size_t)row, vecs, c, h);
#pragma unroll
  for (int e = 0; e < NE; ++e) {
    const float s = 1.0f / (1.0f + __expf(-g[e]));
    const float dg = h[e] * u[e] * s * (1.0f + g[e] * (1.0f - s));
    const float du = h[e] * g[e] * s;
    g[e] = dg;
    u[e] = du;
  }
  R::store_round(gu, (size_t)row, 2 * vecs, c, g);
  R::store_round(gu, (size_t)row, 2 * vecs, vecs + c, u);
}

static int launch_swiglu_bwd(const occult_cfg_t& c, void* gu, const void* dh, long long rows, hipStream_t s) {
  if (rows == 0) return OCCULT_OK;
  const int ne = c.dtype == OCCULT_BF16 ? 8 : 4;
  const long long n = rows * (c.f / ne);
  OCC_REQUIRE((n + 255) / 256 < (1ll << 31), OCCULT_EINVAL, "SwiGLU backward grid too large");
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (c.dtype == OCCULT_BF16) hipLaunchKernelGGL(swiglu_bwd_kernel<true>, grid, block, 0, s, gu, dh, rows, c.f);
  else hipLaunchKernelGGL(swiglu_bwd_kernel<false>, grid, block, 0, s, gu, dh, rows, c.f);
  OCC_LAUNCH_CHECK("swiglu_bwd_kernel");
  return OCCULT_OK;
}

// in [n][R][C] -> out[m][c][col0 + r]
static int launch_transpose(const occult_cfg_t& c, const void* in, void* out, int R, int C, long long out_mat_stride,
                            int out_ld, int col0, hipStream_t s) {
  const dim3 grid((C + 63) / 64, (R + 63) / 64, c.E + c.S), block(256);
  if (c.dtype == OCCULT_BF16)   // d and f are multiples of 8 (16-byte rows), so every vector is whole and aligned
    hipLaunchKernelGGL(transpose16_kernel, grid, block, 0, s, static_cast<const unsigned short*>(in),
                       static_cast<unsigned short*>(out), R, C, out_mat_stride, out_ld, col0);
  else
    hipLaunchKernelGGL(transpose_kernel<float>, grid, block, 0, s, static_cast<const float*>(in),
                       static_cast<float*>(out), R, C, out_mat_stride, out_ld, col0);
  OCC_LAUNCH_CHECK("transpose_kernel");
  return OCCULT_OK;
}

static int launch_transposes(const occult_cfg_t& c, const occult_weights_t* w, void* w_down_t, void* w_gu_t,
                             hipStream_t s) {
  const long long mat = (long long)c.f * c.d;
  // w_down [n][d][f] -> [n][f][d]
  int rc = launch_transpose(c, w->w_down, w_down_t, c.d, c.f, mat, c.d, 0, s);
  if (rc) return rc;
  // w_gate, w_up [n][f][d] -> [n][d][2f], gate in columns [0, f), up in [f, 2f)
  rc = launch_transpose(c, w->w_gate, w_gu_t, c.f, c.d, 2 * mat, 2 * c.f, 0, s);
  if (rc) return rc;
  return launch_transpose(c, w->w_up, w_gu_t, c.f, c.d, 2 * mat, 2 * c.f, c.f, s);
}

static int check_ffn_shapes(const occult_cfg_t& c) {
  const int es = elem_size(c);
  OCC_REQUIRE(((size_t)c.d * es) % 16 == 0 && ((size_t)c.f * es) % 16 == 0, OCCULT_EALIGN,
              "rows of d=%d or f=%d elements are not multiples of 16 bytes", c.d, c.f);
  if (c.dtype == OCCULT_BF16)
    OCC_REQUIRE(c.d % 64 == 0 && c.f % 64 == 0, OCCULT_ESHAPE,
                "bf16 path needs d and f to be multiples of 64 (d=%d, f=%d)", c.d, c.f);
  return OCCULT_OK;
}

}  // namespace occult

using namespace occult;

extern "C" int occult_transpose_weights(const occult_cfg_t* cfg, const occult_weights_t* weights, void* w_down_t,
                                        void* w_gu_t, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  OCC_REQUIRE(weights && weights->w_gate && weights->w_up && weights->w_down, OCCULT_ENULLPTR,
              "weights or one of its tensors is NULL");
  OCC_REQUIRE(w_down_t && w_gu_t, OCCULT_ENULLPTR, "w_down_t or w_gu_t is NULL");
  OCC_REQUIRE((c.E + c.S) <= 65535, OCCULT_EINVAL, "too many weight matrices");
  const int es = elem_size(c);
  OCC_REQUIRE(((size_t)c.d * es) % 16 == 0 && ((size_t)c.f * es) % 16 == 0, OCCULT_EALIGN,
              "rows of d=%d or f=%d elements are not multiples of 16 bytes", c.d, c.f);
  OCC_REQUIRE(aligned16(weights->w_gate) && aligned16(weights->w_up) && aligned16(weights->w_down) &&
                  aligned16(w_down_t) && aligned16(w_gu_t),
              OCCULT_EALIGN, "a buffer is not 16-byte aligned");
  return launch_transposes(c, weights, w_down_t, w_gu_t, static_cast<hipStream_t>(stream));
}

extern "C" int occult_expert_ffn_backward(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                          const void* x, const occult_weights_t* weights, const void* w_down_t,
                                          const void* w_gu_t, const void* epd_dy, const void* dy, void* epd_gu,
                                          void* epd_dh, void* epd_dx, void* gu_shared, void* dh_shared,
                                          void* dx_shared, int gu_saved, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(plan && plan->exp_offset && plan->pos_expert && plan->epd_sfd_row, OCCULT_ENULLPTR,
              "plan or one of its tables is NULL");
  OCC_REQUIRE(weights && weights->w_gate && weights->w_up && w_down_t && w_gu_t, OCCULT_ENULLPTR,
              "weights, w_down_t or w_gu_t is NULL");
  OCC_REQUIRE(sfd_x && epd_dy && epd_gu && epd_dh && epd_dx, OCCULT_ENULLPTR,
              "sfd_x, epd_dy, epd_gu, epd_dh or epd_dx is NULL");
  if (c.S > 0)
    OCC_REQUIRE(x && dy && gu_shared && dh_shared && dx_shared, OCCULT_ENULLPTR,
                "x, dy, gu_shared, dh_shared or dx_shared is NULL with S=%d", c.S);
  rc = check_ffn_shapes(c);
  if (rc) return rc;
  OCC_REQUIRE(aligned16(sfd_x) && aligned16(x) && aligned16(weights->w_gate) && aligned16(weights->w_up) &&
                  aligned16(w_down_t) && aligned16(w_gu_t) && aligned16(epd_dy) && aligned16(dy) && aligned16(epd_gu) &&
                  aligned16(epd_dh) && aligned16(epd_dx) && aligned16(gu_shared) && aligned16(dh_shared) &&
                  aligned16(dx_shared),
              OCCULT_EALIGN, "a buffer is not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n_epd = c.T * c.k;
  const long long mat = (long long)c.f * c.d;

  // ---- routed experts: groups = placement positions over the EPD rows -----------------------
  GemmArgs base{};
  base.grp_offset = plan->exp_offset; base.grp_widx = plan->pos_expert; base.w_base = 0;
  base.ngroups = c.E; base.M = 0;
  OCC_REQUIRE(gu_saved == 0 || gu_saved == 1, OCCULT_EINVAL, "gu_saved=%d must be 0 or 1", gu_saved);
  if (!gu_saved) {   // g | u: the forward's first product without its SwiGLU epilogue, gate then up
    GemmArgs a = base;
    a.A = sfd_x; a.lda = c.d; a.a_rows = plan->epd_sfd_row; a.a_rows_total = sfd_rows_max(c);
    a.b_group_stride = mat; a.ldb = c.d; a.kseg = c.d;
    a.C = epd_gu; a.ldc = 2 * c.f; a.N = c.f; a.K = c.d;
    a.B = weights->w_gate; a.c_col0 = 0;
    rc = launch_gemm(c, a, false, n_epd, s);
    if (rc) return rc;
    a.B = weights->w_up; a.c_col0 = c.f;
    rc = launch_gemm(c, a, false, n_epd, s);
    if (rc) return rc;
  }
  {   // dh = epd_dy W_down: contraction over d against the transposed down projection [f][d]
    GemmArgs a = base;
    a.A = epd_dy; a.lda = c.d; a.a_rows = nullptr; a.a_rows_total = n_epd;
    a.B = w_down_t; a.b_group_stride = mat; a.ldb = c.d; a.kseg = c.d;
    a.C = epd_dh; a.ldc = c.f; a.c_col0 = 0; a.N = c.f; a.K = c.d;
    rc = launch_gemm(c, a, false, n_epd, s);
    if (rc) return rc;
  }
  rc = launch_swiglu_bwd(c, epd_gu, epd_dh, n_epd, s);
  if (rc) return rc;
  {   // epd_dx = [dg | du] [W_gate^T | W_up^T]^T: one product over K = 2f
    GemmArgs a = base;
    a.A = epd_gu; a.lda = 2 * c.f; a.a_rows = nullptr; a.a_rows_total = n_epd;
    a.B = w_gu_t; a.b_group_stride = 2 * mat; a.ldb = 2 * c.f; a.kseg = 2 * c.f;
    a.C = epd_dx; a.ldc = c.d; a.c_col0 = 0; a.N = c.d; a.K = 2 * c.f;
    rc = launch_gemm(c, a, false, n_epd, s);
    if (rc) return rc;
  }
  if (c.S == 0) return OCCULT_OK;

  // ---- shared experts: S uniform groups over the T rows of x; every token with weight 1 ------
  GemmArgs sh{};
  sh.grp_offset = nullptr; sh.grp_widx = nullptr; sh.w_base = c.E; sh.ngroups = c.S; sh.M = c.T;
  sh.a_rows = nullptr; sh.a_rows_total = c.T;
  if (!gu_saved) {
    GemmArgs a = sh;
    a.A = x; a.lda = c.d;
    a.b_group_stride = mat; a.ldb = c.d; a.kseg = c.d;
    a.C = gu_shared; a.ldc = c.S * 2 * c.f; a.c_group_cols = 2 * c.f; a.N = c.f; a.K = c.d;
    a.B = weights->w_gate; a.c_col0 = 0;
    rc = launch_gemm(c, a, false, c.T * c.S, s);
    if (rc) return rc;
    a.B = weights->w_up; a.c_col0 = c.f;
    rc = launch_gemm(c, a, false, c.T * c.S, s);
    if (rc) return rc;
  }
  {
    GemmArgs a = sh;
    a.A = dy; a.lda = c.d;
    a.B = w_down_t; a.b_group_stride = mat; a.ldb = c.d; a.kseg = c.d;
    a.C = dh_shared; a.ldc = c.S * c.f; a.c_col0 = 0; a.c_group_cols = c.f; a.N = c.f; a.K = c.d;
    rc = launch_gemm(c, a, false, c.T * c.S, s);
    if (rc) return rc;
  }
  rc = launch_swiglu_bwd(c, gu_shared, dh_shared, (long long)c.T * c.S, s);
  if (rc) return rc;
  {   // one product whose K dimension walks the S transposed gate | up matrices
    GemmArgs a = sh;
    a.ngroups = 1;
    a.A = gu_shared; a.lda = c.S * 2 * c.f;
    a.B = w_gu_t; a.b_group_stride = 2 * mat; a.ldb = 2 * c.f; a.kseg = 2 * c.f;
    a.C = dx_shared; a.ldc = c.d; a.c_col0 = 0; a.N = c.d; a.K = c.S * 2 * c.f;
    rc = launch_gemm(c, a, false, c.T, s);
    if (rc) return rc;
  }
  return OCCULT_OK;
}
