// occult_coactivation: E x E expert co-activation counts (paper Preliminary, the co-activation
// graph C) and occult_placement_greedy: Algorithm 1 of Sec. 3.2 on the host.
//
// Counting: every token contributes k*k increments.  A block keeps a private E x E int32 tile in
// LDS (64 KiB at E = 128), counts its grid-stride share of tokens there with LDS atomics, and
// flushes the non-zero entries with global integer atomics.  Integer adds commute, so the
// result does not depend on scheduling.  E > 128 counts straight into global memory.
#include "common.h"

#include <algorithm>
#include <vector>

namespace occult {

constexpr int kCoactThreads = 256;
constexpr int kCoactLdsMaxE = 128;

__global__ void fill_i32(int32_t* __restrict__ p, size_t n, int32_t v) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = v;
}

// OVERWRITE: the launch is a single block that owns the whole result: its LDS tile is stored, not added, and C
// needs no clearing beforehand.
template <bool OVERWRITE>
__global__ __launch_bounds__(kCoactThreads) void coact_lds_kernel(const int32_t* __restrict__ ids, int T,
                                                                  int k, int E, int32_t* __restrict__ C) {
  extern __shared__ int s_c[];   // [E*E]
  for (int i = threadIdx.x; i < E * E; i += kCoactThreads) s_c[i] = 0;
  __syncthreads();
  // C is symmetric: only the cells on and above the diagonal are counted in LDS (the LDS atomics are what this kernel
  // spends its time on), the flush mirrors them.  A pair of slots naming the same expert adds 2 to its diagonal cell,
  // as the two ordered pairs would.
  for (int t = blockIdx.x * kCoactThreads + threadIdx.x; t < T; t += gridDim.x * kCoactThreads) {
    const int32_t* row = ids + (size_t)t * k;
    for (int a = 0; a < k; ++a) {
      const int ea = row[a];
      atomicAdd(&s_c[ea * E + ea], 1);
      for (int b = a + 1; b < k; ++b) {
        const int eb = row[b];
        const int lo = min(ea, eb), hi = max(ea, eb);
        atomicAdd(&s_c[lo * E + hi], lo == hi ? 2 : 1);
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < E * E; i += kCoactThreads) {
    const int r = i / E, c = i - r * E;
    const int v = r <= c ? s_c[i] : s_c[c * E + r];
    if (OVERWRITE) C[i] = v;
    else if (v) atomicAdd(&C[i], v);
  }
}

__global__ __launch_bounds__(kCoactThreads) void coact_global_kernel(const int32_t* __restrict__ ids, int T,
                                                                     int k, int E, int32_t* __restrict__ C) {
  for (int t = blockIdx.x * kCoactThreads + threadIdx.x; t < T; t += gridDim.x * kCoactThreads) {
    const int32_t* row = ids + (size_t)t * k;
    for (int a = 0; a < k; ++a) {
      const int ea = row[a];
      for (int b = 0; b < k; ++b) atomicAdd(&C[ea * E + row[b]], 1);
    }
  }
}

}  // namespace occult

using namespace occult;

extern "C" int occult_coactivation(const occult_cfg_t* cfg, const int32_t* ids, int32_t* C, int accumulate,
                                   occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  OCC_REQUIRE(C, OCCULT_ENULLPTR, "C is NULL");
  OCC_REQUIRE(c.T == 0 || ids, OCCULT_ENULLPTR, "ids is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t n = (size_t)c.E * c.E;
  int blocks = (c.T + kCoactThreads - 1) / kCoactThreads;
  if (blocks > 512) blocks = 512;
  const bool single = !accumulate && blocks == 1 && c.E <= kCoactLdsMaxE;   // decode steps: one launch, no clearing
  if (!accumulate && !single) {
    hipLaunchKernelGGL(fill_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, C, n, 0);
    OCC_LAUNCH_CHECK("fill_i32");
  }
  if (c.T == 0) return OCCULT_OK;
  if (single) {
    hipLaunchKernelGGL(coact_lds_kernel<true>, dim3(1), dim3(kCoactThreads), n * sizeof(int), s, ids, c.T, c.k, c.E, C);
    OCC_LAUNCH_CHECK("coact_lds_kernel");
  } else if (c.E <= kCoactLdsMaxE) {
    hipLaunchKernelGGL(coact_lds_kernel<false>, dim3(blocks), dim3(kCoactThreads), n * sizeof(int), s, ids, c.T, c.k,
                       c.E, C);
    OCC_LAUNCH_CHECK("coact_lds_kernel");
  } else {
    hipLaunchKernelGGL(coact_global_kernel, dim3(blocks), dim3(kCoactThreads), 0, s, ids, c.T, c.k, c.E, C);
    OCC_LAUNCH_CHECK("coact_global_kernel");
  }
  return OCCULT_OK;
}

// Host: greedy partition of the experts into D groups of G (Algorithm 1).  Candidates of one
// step share their divisor, so integer sums of C are compared; the diagonal never takes part.
// Two running score vectors replace the per-step sums over lists: to_placed[e] = summed count
// between e and every expert placed so far, to_device[e] = the same for the device being filled;
// a push adds one row of C to each (O(E^2) in total).
extern "C" int occult_placement_greedy(const int32_t* C_host, int32_t E, int32_t D, int32_t* L_host,
                                       int32_t* expert_pos_host) {
  OCC_REQUIRE(C_host && L_host && expert_pos_host, OCCULT_ENULLPTR, "a pointer is NULL");
  OCC_REQUIRE(E >= 1 && E <= OCCULT_MAX_E && D >= 1 && D <= OCCULT_MAX_D, OCCULT_EINVAL,
              "E=%d or D=%d out of range", E, D);
  OCC_REQUIRE(E % D == 0, OCCULT_ESHAPE, "E=%d is not divisible by D=%d", E, D);
  const int G = E / D;
  OCC_REQUIRE(G >= 2, OCCULT_ESHAPE, "placement needs at least 2 experts per device (E/D=%d)", G);
  std::vector<int64_t> to_placed(E, 0), to_device(E, 0);
  std::vector<char> free_expert(E, 1);
  int next_pos = 0;
  auto push = [&](int e) {
    const int32_t* row = C_host + (size_t)e * E;
    for (int j = 0; j < E; ++j) {
      to_placed[j] += row[j];
      to_device[j] += row[j];
    }
    free_expert[e] = 0;
    L_host[next_pos] = e;
    expert_pos_host[e] = next_pos++;
  };
  // best free expert under `score`; sign = +1 takes the largest, -1 the smallest; first index wins ties
  auto pick = [&](const std::vector<int64_t>& score, int sign) {
    int best = -1;
    for (int e = 0; e < E; ++e)
      if (free_expert[e] && (best < 0 || sign * score[e] > sign * score[best])) best = e;
    return best;
  };
  for (int dev = 0; dev < D; ++dev) {
    std::fill(to_device.begin(), to_device.end(), 0);
    if (dev == 0) {
      // the most co-activated pair above the diagonal, row-major scan: first maximum = smallest (i, j)
      size_t arg = 1;
      for (int i = 0; i < E; ++i)
        for (int j = i + 1; j < E; ++j)
          if (C_host[(size_t)i * E + j] > C_host[arg]) arg = (size_t)i * E + j;
      push((int)(arg / E));
      push((int)(arg % E));
    } else {
      push(pick(to_placed, -1));
    }
    while (next_pos < (dev + 1) * G) push(pick(to_device, +1));
  }
  return OCCULT_OK;
}

// Host: the placement's collaboration statistics (Sec. 3.2) from co-activation counts.
extern "C" int occult_collaboration_stats(const int32_t* C_host, int32_t E, int32_t D,
                                          const int32_t* expert_pos_host, double* c_intra_host,
                                          double* c_inter_host, double* intra_fraction_host) {
  OCC_REQUIRE(C_host && c_intra_host && c_inter_host && intra_fraction_host, OCCULT_ENULLPTR, "a pointer is NULL");
  OCC_REQUIRE(E >= 1 && E <= OCCULT_MAX_E && D >= 1 && D <= OCCULT_MAX_D, OCCULT_EINVAL,
              "E=%d or D=%d out of range", E, D);
  OCC_REQUIRE(E % D == 0, OCCULT_ESHAPE, "E=%d is not divisible by D=%d", E, D);
  const int G = E / D;
  std::vector<int> dev_of(E);
  for (int e = 0; e < E; ++e) {
    const int pos = expert_pos_host ? expert_pos_host[e] : e;
    OCC_REQUIRE(pos >= 0 && pos < E, OCCULT_EINVAL, "expert_pos[%d]=%d out of range", e, pos);
    dev_of[e] = pos / G;
  }
  // block sums of the off-diagonal counts per ordered device pair, and the largest off-diagonal count
  std::vector<int64_t> block((size_t)D * D, 0);
  int64_t top = 0;
  for (int i = 0; i < E; ++i)
    for (int j = 0; j < E; ++j) {
      if (i == j) continue;
      const int64_t v = C_host[(size_t)i * E + j];
      block[(size_t)dev_of[i] * D + dev_of[j]] += v;
      if (v > top) top = v;
    }
  int64_t same = 0, all = 0;
  for (int a = 0; a < D; ++a)
    for (int b = 0; b < D; ++b) {
      all += block[(size_t)a * D + b];
      if (a == b) same += block[(size_t)a * D + b];
    }
  *intra_fraction_host = all > 0 ? (double)same / (double)all : 0.0;
  const double scale = top > 0 ? 1.0 / (double)top : 0.0;          // P = C / largest off-diagonal count
  for (int a = 0; a < D; ++a) {
    const double pairs = (double)G * (G - 1);                      // ordered pairs i != j on one device
    c_intra_host[a] = G > 1 ? (double)block[(size_t)a * D + a] * scale / pairs : 0.0;
    for (int b = 0; b < D; ++b)
      c_inter_host[(size_t)a * D + b] = a == b ? 0.0 : (double)block[(size_t)a * D + b] * scale / ((double)G * G);
  }
  return OCCULT_OK;
}
