// occult_dispatch: ORI -> SFD pack (paper App. A.2 "Dispatch"; Sec. 3.1: one replica of a token
// per distinct destination device).
//
// The printed kernel walks (device, token-tile) pairs and so reads every token row once per
// device.  Here the loop is token-major: a wavefront reads row t once with 16-byte lane loads,
// keeps it in registers, and stores it to each of the token's <= min(k, D) SFD rows, so the
// HBM traffic is (1 + c_t) rows per token.  Pure copy: bandwidth bound.
#include "common.h"

namespace occult {

constexpr int kDispWaves = 4;   // waves (tokens in flight) per block

// VPL = 16-byte vectors per lane; row_vecs = d * es / 16 <= 64 * VPL
template <int VPL>
__global__ __launch_bounds__(kDispWaves * 64) void dispatch_kernel(
    const u32x4* __restrict__ x, u32x4* __restrict__ sfd_x, const int32_t* __restrict__ tok_sfd_row,
    int T, int D, int row_vecs) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kDispWaves + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * kDispWaves;
  for (int t = wave; t < T; t += nwaves) {
    u32x4 v[VPL];
    const u32x4* src = x + (size_t)t * row_vecs;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      const int c = lane + 64 * i;
      if (c < row_vecs) v[i] = __builtin_nontemporal_load(src + c);
    }
    // the token's D destination rows in one wave-wide load (D <= 64), then broadcast one by one
    const int rl = lane < D ? tok_sfd_row[(size_t)t * D + lane] : -1;
    for (int j = 0; j < D; ++j) {
      const int r = __builtin_amdgcn_readlane(rl, j);
      if (r < 0) continue;
      u32x4* dst = sfd_x + (size_t)r * row_vecs;
#pragma unroll
      for (int i = 0; i < VPL; ++i) {
        const int c = lane + 64 * i;
        if (c < row_vecs) __builtin_nontemporal_store(v[i], dst + c);
      }
    }
  }
}

// rows longer than 64 * 8 vectors (8 KiB): plain strided loop, row re-read per destination
__global__ __launch_bounds__(kDispWaves * 64) void dispatch_kernel_long(
    const u32x4* __restrict__ x, u32x4* __restrict__ sfd_x, const int32_t* __restrict__ tok_sfd_row,
    int T, int D, int row_vecs) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kDispWaves + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * kDispWaves;
  for (int t = wave; t < T; t += nwaves) {
    const u32x4* src = x + (size_t)t * row_vecs;
    for (int j = 0; j < D; ++j) {
      const int r = tok_sfd_row[(size_t)t * D + j];
      if (r < 0) continue;
      u32x4* dst = sfd_x + (size_t)r * row_vecs;
      for (int c = lane; c < row_vecs; c += 64) dst[c] = src[c];
    }
  }
}

// routing metadata of every dispatched row: one thread per (token, device, slot)
__global__ __launch_bounds__(256) void dispatch_meta_kernel(const int32_t* __restrict__ ids, const float* __restrict__ w,
                                                            const int32_t* __restrict__ tok_sfd_row, int T, int D, int k,
                                                            int32_t* __restrict__ sfd_ids, float* __restrict__ sfd_w) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)T * D * k) return;
  const int s = (int)(i % k);
  const size_t td = i / k;   // token * D + device
  const int r = tok_sfd_row[td];
  if (r < 0) return;
  const size_t t = td / D;
  sfd_ids[(size_t)r * k + s] = ids[t * k + s];
  sfd_w[(size_t)r * k + s] = w[t * k + s];
}

}  // namespace occult

using namespace occult;

extern "C" int occult_dispatch_meta(const occult_cfg_t* cfg, const occult_plan_t* plan, const int32_t* ids,
                                    const float* w, int32_t* sfd_ids, float* sfd_w, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(plan && plan->tok_sfd_row, OCCULT_ENULLPTR, "plan or plan->tok_sfd_row is NULL");
  OCC_REQUIRE(ids && w && sfd_ids && sfd_w, OCCULT_ENULLPTR, "ids, w, sfd_ids or sfd_w is NULL");
  const size_t n = (size_t)c.T * c.D * c.k;
  OCC_REQUIRE((n + 255) / 256 < (1ull << 31), OCCULT_EINVAL, "T*D*k too large for one launch");
  hipLaunchKernelGGL(dispatch_meta_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), ids, w, plan->tok_sfd_row, c.T, c.D, c.k, sfd_ids, sfd_w);
  OCC_LAUNCH_CHECK("dispatch_meta_kernel");
  return OCCULT_OK;
}

extern "C" int occult_dispatch(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* x,
                               void* sfd_x, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(plan && plan->tok_sfd_row, OCCULT_ENULLPTR, "plan or plan->tok_sfd_row is NULL");
  OCC_REQUIRE(x && sfd_x, OCCULT_ENULLPTR, "x or sfd_x is NULL");
  const size_t row_bytes = (size_t)c.d * elem_size(c);
  OCC_REQUIRE(row_bytes % 16 == 0, OCCULT_EALIGN, "row of %zu bytes is not a multiple of 16", row_bytes);
  OCC_REQUIRE(aligned16(x) && aligned16(sfd_x), OCCULT_EALIGN, "x or sfd_x is not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int row_vecs = (int)(row_bytes / 16);
  const int vpl = (row_vecs + 63) / 64;
  const int blocks = (c.T + kDispWaves - 1) / kDispWaves;
  const dim3 grid(blocks), block(kDispWaves * 64);
  const u32x4* xs = static_cast<const u32x4*>(x);
  u32x4* ds = static_cast<u32x4*>(sfd_x);
#define OCC_DISP(N) \
  hipLaunchKernelGGL(dispatch_kernel<N>, grid, block, 0, s, xs, ds, plan->tok_sfd_row, c.T, c.D, row_vecs)
  if (vpl <= 1) OCC_DISP(1);
  else if (vpl <= 2) OCC_DISP(2);
  else if (vpl <= 4) OCC_DISP(4);
  else if (vpl <= 8) OCC_DISP(8);
  else
    hipLaunchKernelGGL(dispatch_kernel_long, grid, block, 0, s, xs, ds, plan->tok_sfd_row, c.T, c.D, row_vecs);
#undef OCC_DISP
  OCC_LAUNCH_CHECK("dispatch_kernel");
  return OCCULT_OK;
}
