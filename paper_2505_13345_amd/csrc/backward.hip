// Backward pass of the layer's data movement and of the routing weights.
//
// The paper trains through the layer (Introduction: the sparse matrix multiplication serves the
// forward and the backward pass; Sec. 4, Training) and prints no backward algorithm.  Every
// forward data-movement step is linear in the hidden rows, so its gradient is the transposed map
// on the same plan (Sec. 3.1 re-index matrices):
//   combine, stage 2   y[t] += sfd_y[r(t, j)]            ->  sfd_dy[r(t, j)] = dy[t]     (a dispatch of dy)
//   combine, stage 1   sfd_y[r] += gate_q * epd_y[q]     ->  epd_dy[q] = gate_q * sfd_dy[r],
//                                                            d gate_q = <sfd_dy[r], epd_y[q]>
//   row gather + dispatch                                ->  occult_dispatch_backward (combine.hip):
//                                                            the two-stage sum with unit weights
// so both backward exchanges again carry one row per (token, device).
//
// combine_bwd_kernel: one wavefront per token, like the forward combine.  Lane s < k looks up
// slot s of its token (expert -> placement position -> device -> SFD row -> the EPD row of that
// position in the row's merge list); the wave then keeps dy[t] in registers and, slot by slot,
// writes the scaled row and reduces the dot product.  Traffic per token: one ORI row in, k EPD
// rows out, k EPD rows in (only if gate gradients are asked for).
#include "common.h"

namespace occult {

constexpr int kBwdWaves = 4;

__device__ __forceinline__ float wave_sum_all(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ float wave_max_all(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

template <bool BF16, int VPL>
__global__ __launch_bounds__(kBwdWaves * 64) void combine_bwd_kernel(
    const void* __restrict__ dy, const void* __restrict__ epd_y, void* __restrict__ epd_dy, float* __restrict__ dw,
    const int32_t* __restrict__ ids, const int32_t* __restrict__ expert_pos,
    const int32_t* __restrict__ tok_sfd_row, const int32_t* __restrict__ sfd_epd_rows,
    const int32_t* __restrict__ exp_offset, const float* __restrict__ epd_gate, int T, int k, int D, int G,
    int M1, int row_vecs) {
  using R = Row<BF16>;
  constexpr int NE = R::kElems;
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kBwdWaves + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * kBwdWaves;
  for (int t = wave; t < T; t += nwaves) {
    // slot lookup, one slot per lane (k <= 32)
    int my_q = -1;
    float my_g = 0.0f;
    if (lane < k) {
      const int e = ids[(size_t)t * k + lane];
      const int P = expert_pos ? expert_pos[e] : e;
      const int r = tok_sfd_row[(size_t)t * D + P / G];
      if (r >= 0) {
        const int lo = exp_offset[P], hi = exp_offset[P + 1];
        for (int m = 0; m < M1; ++m) {
          const int q = sfd_epd_rows[(size_t)r * M1 + m];
          if (q >= lo && q < hi) my_q = q;   // -1 padding is never inside [lo, hi)
        }
      }
      if (my_q >= 0) my_g = epd_gate[my_q];
    }
    float my_dw = 0.0f;
    // rows longer than 64 * VPL vectors are done in column chunks; the slot lookup stays in registers
    for (int cbase = 0; cbase < row_vecs; cbase += 64 * VPL) {
      float g_row[VPL][NE];
#pragma unroll
      for (int i = 0; i < VPL; ++i) {
        const int c = cbase + lane + 64 * i;
        if (c < row_vecs) {
          R::load(dy, (size_t)t, row_vecs, c, g_row[i]);
        } else {
#pragma unroll
          for (int e = 0; e < NE; ++e) g_row[i][e] = 0.0f;
        }
      }
      for (int s = 0; s < k; ++s) {
        const int q = __builtin_amdgcn_readlane(my_q, s);
        if (q < 0) continue;   // a plan that does not belong to these ids: nothing to address
        const float g = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_g), s));
        float dot = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
          const int c = cbase + lane + 64 * i;
          if (c < row_vecs) {
            if (dw) {
              float v[NE];
              R::load(epd_y, (size_t)q, row_vecs, c, v);
#pragma unroll
              for (int e = 0; e < NE; ++e) dot = fmaf(g_row[i][e], v[e], dot);
            }
            if (epd_dy) {
              float o[NE];
#pragma unroll
              for (int e = 0; e < NE; ++e) o[e] = g * g_row[i][e];
              R::store_round(epd_dy, (size_t)q, row_vecs, c, o);
            }
          }
        }
        if (dw) {
          dot = wave_sum_all(dot);
          if (lane == s) my_dw += dot;
        }
      }
    }
    if (dw && lane < k) dw[(size_t)t * k + lane] = my_dw;
  }
}

// Gradient of the gate values with respect to the router scores (paper Eq. 1: Softmax over all E
// experts, the values at the k selected ones, divided by their sum when renorm).  One wavefront
// per token, expert e on lane e % 64.
template <int EPL>
__global__ __launch_bounds__(256) void route_bwd_kernel(const float* __restrict__ logits, const int32_t* __restrict__ ids,
                                                        const float* __restrict__ dw, float* __restrict__ dlogits,
                                                        int T, int E, int k, int renorm) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;   // wave-uniform
  float l[EPL], p[EPL], a[EPL];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = lane + 64 * i;
    l[i] = e < E ? logits[(size_t)t * E + e] : -INFINITY;
    mx = fmaxf(mx, l[i]);
  }
  mx = wave_max_all(mx);
  float z = 0.0f;
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    p[i] = lane + 64 * i < E ? expf(l[i] - mx) : 0.0f;
    z += p[i];
  }
  z = wave_sum_all(z);
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    p[i] /= z;
    a[i] = 0.0f;
  }
  // gradient with respect to the selected softmax values, scattered to the experts' lanes
  const int my_id = lane < k ? ids[(size_t)t * k + lane] : -1;
  const float my_gw = lane < k ? dw[(size_t)t * k + lane] : 0.0f;
  bool sel[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) sel[i] = false;
  for (int s = 0; s < k; ++s) {
    const int id = __builtin_amdgcn_readlane(my_id, s);
    const float gw = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_gw), s));
#pragma unroll
    for (int i = 0; i < EPL; ++i)
      if (lane + 64 * i == id) {
        a[i] = gw;
        sel[i] = true;
      }
  }
  if (renorm) {
    float zs = 0.0f, dot = 0.0f;
#pragma unroll
    for (int i = 0; i < EPL; ++i)
      if (sel[i]) {
        zs += p[i];
        dot = fmaf(a[i], p[i], dot);
      }
    zs = wave_sum_all(zs);
    dot = wave_sum_all(dot) / zs;   // sum_s dw_s * w_s
#pragma unroll
    for (int i = 0; i < EPL; ++i) a[i] = sel[i] ? (a[i] - dot) / zs : 0.0f;
  }
  float inner = 0.0f;
#pragma unroll
  for (int i = 0; i < EPL; ++i) inner = fmaf(a[i], p[i], inner);
  inner = wave_sum_all(inner);
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = lane + 64 * i;
    if (e < E) dlogits[(size_t)t * E + e] = p[i] * (a[i] - inner);
  }
}

}  // namespace occult

using namespace occult;

extern "C" int occult_combine_backward(const occult_cfg_t* cfg, const occult_plan_t* plan, const int32_t* ids,
                                       const void* dy, const void* epd_y, void* sfd_dy, void* epd_dy, float* dw,
                                       occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(plan && plan->tok_sfd_row && plan->sfd_epd_rows && plan->exp_offset && plan->epd_gate, OCCULT_ENULLPTR,
              "plan or one of its tables is NULL");
  OCC_REQUIRE(ids && dy, OCCULT_ENULLPTR, "ids or dy is NULL");
  OCC_REQUIRE(dw == nullptr || epd_y != nullptr, OCCULT_ENULLPTR, "dw needs epd_y");
  if (sfd_dy) {   // transposed stage 2: every SFD row receives its token's gradient
    rc = occult_dispatch(cfg, plan, dy, sfd_dy, stream);
    if (rc) return rc;
  }
  if (!epd_dy && !dw) return OCCULT_OK;
  const size_t row_bytes = (size_t)c.d * elem_size(c);
  OCC_REQUIRE(row_bytes % 16 == 0, OCCULT_EALIGN, "row of %zu bytes is not a multiple of 16", row_bytes);
  OCC_REQUIRE(aligned16(dy) && aligned16(epd_y) && aligned16(epd_dy), OCCULT_EALIGN, "a buffer is not 16-byte aligned");
  const int row_vecs = (int)(row_bytes / 16);
  const int vpl = (row_vecs + 63) / 64;   // beyond 8 the kernel walks the row in chunks of 8 KiB
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid((c.T + kBwdWaves - 1) / kBwdWaves), block(kBwdWaves * 64);
#define OCC_CBWD(B, N)                                                                                       \
  hipLaunchKernelGGL((combine_bwd_kernel<B, N>), grid, block, 0, s, dy, epd_y, epd_dy, dw, ids, c.expert_pos, \
                     plan->tok_sfd_row, plan->sfd_epd_rows, plan->exp_offset, plan->epd_gate, c.T, c.k, c.D,  \
                     c.E / c.D, merge_width(c), row_vecs)
  if (c.dtype == OCCULT_BF16) {
    if (vpl <= 1) OCC_CBWD(true, 1);
    else if (vpl <= 2) OCC_CBWD(true, 2);
    else if (vpl <= 4) OCC_CBWD(true, 4);
    else OCC_CBWD(true, 8);
  } else {
    if (vpl <= 1) OCC_CBWD(false, 1);
    else if (vpl <= 2) OCC_CBWD(false, 2);
    else if (vpl <= 4) OCC_CBWD(false, 4);
    else OCC_CBWD(false, 8);
  }
#undef OCC_CBWD
  OCC_LAUNCH_CHECK("combine_bwd_kernel");
  return OCCULT_OK;
}

extern "C" int occult_route_backward(const occult_cfg_t* cfg, const float* logits, const int32_t* ids, const float* dw,
                                     float* dlogits, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(logits && ids && dw && dlogits, OCCULT_ENULLPTR, "logits, ids, dw or dlogits is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid((c.T + 3) / 4), block(256);
  const int epl = (c.E + 63) / 64;
#define OCC_RBWD(N) \
  hipLaunchKernelGGL(route_bwd_kernel<N>, grid, block, 0, s, logits, ids, dw, dlogits, c.T, c.E, c.k, c.renorm)
  if (epl <= 1) OCC_RBWD(1);
  else if (epl <= 2) OCC_RBWD(2);
  else OCC_RBWD(4);
#undef OCC_RBWD
  OCC_LAUNCH_CHECK("route_bwd_kernel");
  return OCCULT_OK;
}
