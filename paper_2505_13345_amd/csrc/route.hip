// occult_route: softmax top-k gating with optional collaboration pruning
// (paper Eq. 1; Section 3.3, routing-score-based pruning).
//
// One 64-lane wavefront per token.  Lane l holds the scores of experts l, l+64, l+128, l+192
// (E <= 256), so a row of scores is read with coalesced loads and a selection round is a
// per-lane best followed by a 6-step butterfly arg-max over the wave.  Selection compares raw
// scores (softmax is monotone): larger first, equal -> lower expert index.
//
// The pruning decision of mode 1 compares per-device sums of exp(score - max); those sums are
// taken in one fixed float32 sequence (exp_ref below: separately rounded multiplies and adds,
// no contraction into FMAs) so that a CPU restatement of the same text reaches the same bits.
#include "common.h"

#include <limits.h>
#include <math.h>

// every float operation in this file is rounded on its own
#pragma clang fp contract(off)

namespace occult {

__device__ __forceinline__ float exp_ref(float z) {
  // z <= 0.  z < -80 -> 0.  n = rint(z*log2e); r = (z - n*ln2_hi) - n*ln2_lo; degree-7 Taylor
  // polynomial by Horner; result scaled by 2^n through the exponent bits.
  const float kLog2e = 1.4426950408889634f;
  const float kLn2Hi = 0.693359375f;
  const float kLn2Lo = -2.12194440054690583e-4f;
  const float zc = fmaxf(z, -80.0f);
  const float n = rintf(zc * kLog2e);
  float r = zc - n * kLn2Hi;
  r = r - n * kLn2Lo;
  float p = 1.0f / 5040.0f;
  p = p * r + 1.0f / 720.0f;
  p = p * r + 1.0f / 120.0f;
  p = p * r + 1.0f / 24.0f;
  p = p * r + 1.0f / 6.0f;
  p = p * r + 0.5f;
  p = p * r + 1.0f;
  p = p * r + 1.0f;
  const float scale = __int_as_float(((int)n + 127) << 23);
  const float out = p * scale;
  return z < -80.0f ? 0.0f : out;
}

__device__ __forceinline__ void wave_argmax(float& v, int& i) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(v, off, 64);
    const int oi = __shfl_xor(i, off, 64);
    const bool take = (ov > v) || (ov == v && oi < i);
    v = take ? ov : v;
    i = take ? oi : i;
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

constexpr int kRouteWavesPerBlock = 4;

template <int EPL>  // experts per lane = ceil(E / 64)
__global__ __launch_bounds__(kRouteWavesPerBlock * 64) void route_kernel(
    const float* __restrict__ logits, int T, int E, int k, int D, int G,
    const int32_t* __restrict__ expert_pos, int n_d, int prune_mode, int renorm,
    int32_t* __restrict__ ids, float* __restrict__ w) {
  __shared__ int s_dev[OCCULT_MAX_E];
  for (int e = threadIdx.x; e < E; e += blockDim.x)
    s_dev[e] = (expert_pos ? expert_pos[e] : e) / G;
  __syncthreads();

  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * kRouteWavesPerBlock + (threadIdx.x >> 6);
  if (t >= T) return;   // whole wave leaves together; no barrier follows

  const float kNegInf = -INFINITY;
  float v0[EPL];   // the token's scores as read (with -0.0 folded onto +0.0)
  float v[EPL];    // working copy: taken / disallowed entries become -inf
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = lane + 64 * i;
    v0[i] = (e < E) ? (logits[(size_t)t * E + e] + 0.0f) : kNegInf;
    v[i] = v0[i];
  }

  auto select_round = [&](float& bv, int& bi) {
    bv = kNegInf;
    bi = INT_MAX;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const int e = lane + 64 * i;
      // strictly greater keeps the lower index among a lane's equal scores (i ascending)
      if (e < E && (v[i] > bv || bi == INT_MAX)) {
        bv = v[i];
        bi = e;
      }
    }
    wave_argmax(bv, bi);
#pragma unroll
    for (int i = 0; i < EPL; ++i)
      if (lane + 64 * i == bi) v[i] = kNegInf;
  };

  int my_id = 0;       // lane s < k keeps slot s
  float my_v = 0.0f;
  float mx = 0.0f;
  float dev_sum = 0.0f;          // lane j < D: mode-1 score of device j
  unsigned long long kept = 0;   // mode 2: devices kept so far (wave-uniform)
  int n_kept = 0;

  for (int s = 0; s < k; ++s) {
    float bv;
    int bi;
    select_round(bv, bi);
    if (s == 0) mx = bv;
    if (lane == s) {
      my_id = bi;
      my_v = bv;
    }
    if (n_d > 0) {
      const int dev = s_dev[bi];
      if (prune_mode == 1) {
        const float q = exp_ref(bv - mx);
        if (lane == dev) dev_sum = dev_sum + q;   // sequential in slot order
      } else if (!((kept >> dev) & 1ull) && n_kept < n_d) {
        kept |= 1ull << dev;
        ++n_kept;
      }
    }
  }

  if (n_d > 0) {
    if (prune_mode == 1) {
      float sv = (lane < D) ? dev_sum : kNegInf;
      kept = 0;
      for (int r = 0; r < n_d; ++r) {
        float bv = sv;
        int bi = (lane < D) ? lane : INT_MAX;
        wave_argmax(bv, bi);
        kept |= 1ull << bi;
        if (lane == bi) sv = kNegInf;
      }
    }
    // second pass: the k best experts on the surviving devices
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const int e = lane + 64 * i;
      const bool ok = (e < E) && ((kept >> s_dev[e < E ? e : 0]) & 1ull);
      v[i] = ok ? v0[i] : kNegInf;
    }
    for (int s = 0; s < k; ++s) {
      float bv;
      int bi;
      select_round(bv, bi);
      if (lane == s) {
        my_id = bi;
        my_v = bv;
      }
    }
  }

  // gate values: softmax over all E experts at the selected ones
  float part = 0.0f;
#pragma unroll
  for (int i = 0; i < EPL; ++i)
    if (lane + 64 * i < E) part += exp_ref(v0[i] - mx);
  const float denom = wave_sum(part);
  float g = (lane < k) ? exp_ref(my_v - mx) / denom : 0.0f;
  if (renorm) {
    const float sel = wave_sum(g);
    g = g / sel;
  }
  if (lane < k) {
    ids[(size_t)t * k + lane] = my_id;
    w[(size_t)t * k + lane] = g;
  }
}

}  // namespace occult

using namespace occult;

extern "C" int occult_route(const occult_cfg_t* cfg, const float* logits, int32_t* ids, float* w,
                            occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(logits && ids && w, OCCULT_ENULLPTR, "logits, ids or w is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int G = c.E / c.D;
  const dim3 grid((c.T + kRouteWavesPerBlock - 1) / kRouteWavesPerBlock), block(kRouteWavesPerBlock * 64);
  const int epl = (c.E + 63) / 64;
#define OCC_ROUTE_LAUNCH(N)                                                                     \
  hipLaunchKernelGGL(route_kernel<N>, grid, block, 0, s, logits, c.T, c.E, c.k, c.D, G,         \
                     c.expert_pos, c.n_d, c.prune_mode, c.renorm, ids, w)
  switch (epl) {
    case 1: OCC_ROUTE_LAUNCH(1); break;
    case 2: OCC_ROUTE_LAUNCH(2); break;
    case 3: OCC_ROUTE_LAUNCH(3); break;
    default: OCC_ROUTE_LAUNCH(4); break;
  }
#undef OCC_ROUTE_LAUNCH
  OCC_LAUNCH_CHECK("route_kernel");
  return OCCULT_OK;
}
