// occult_coactivation: E x E expert co-activation counts (paper Preliminary, the co-activation
// graph C) and occult_placement_greedy: Algorithm 1 of Sec. 3.2 on the host.
//
// Counting: every token contributes k*k increments.  A block keeps a private E x E int32 tile in
// LDS (64 KiB at E = 128), counts its grid-stride share of tokens there with LDS atomics, and
// flushes the non-zero entries with global integer atomics.  Integer adds commute, so the
// result does not depend on scheduling.  E > 128 counts straight into global memory.
#include "common.h"

#include <vector>

namespace occult {

constexpr int kCoactThreads = 256;
constexpr int kCoactLdsMaxE = 128;

__global__ void fill_i32(int32_t* __restrict__ p, size_t n, int32_t v) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = v;
}

__global__ __launch_bounds__(kCoactThreads) void coact_lds_kernel(const int32_t* __restrict__ ids, int T,
                                                                  int k, int E, int32_t* __restrict__ C) {
  extern __shared__ int s_c[];   // [E*E]
  for (int i = threadIdx.x; i < E * E; i += kCoactThreads) s_c[i] = 0;
  __syncthreads();
  for (int t = blockIdx.x * kCoactThreads + threadIdx.x; t < T; t += gridDim.x * kCoactThreads) {
    const int32_t* row = ids + (size_t)t * k;
    for (int a = 0; a < k; ++a) {
      const int ea = row[a];
      for (int b = 0; b < k; ++b) atomicAdd(&s_c[ea * E + row[b]], 1);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < E * E; i += kCoactThreads) {
    const int v = s_c[i];
    if (v) atomicAdd(&C[i], v);
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
  if (!accumulate) {
    hipLaunchKernelGGL(fill_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, C, n, 0);
    OCC_LAUNCH_CHECK("fill_i32");
  }
  if (c.T == 0) return OCCULT_OK;
  int blocks = (c.T + kCoactThreads - 1) / kCoactThreads;
  if (blocks > 512) blocks = 512;
  if (c.E <= kCoactLdsMaxE) {
    hipLaunchKernelGGL(coact_lds_kernel, dim3(blocks), dim3(kCoactThreads), n * sizeof(int), s, ids, c.T, c.k,
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
extern "C" int occult_placement_greedy(const int32_t* C_host, int32_t E, int32_t D, int32_t* L_host,
                                       int32_t* expert_pos_host) {
  OCC_REQUIRE(C_host && L_host && expert_pos_host, OCCULT_ENULLPTR, "a pointer is NULL");
  OCC_REQUIRE(E >= 1 && E <= OCCULT_MAX_E && D >= 1 && D <= OCCULT_MAX_D, OCCULT_EINVAL,
              "E=%d or D=%d out of range", E, D);
  OCC_REQUIRE(E % D == 0, OCCULT_ESHAPE, "E=%d is not divisible by D=%d", E, D);
  const int G = E / D;
  OCC_REQUIRE(G >= 2, OCCULT_ESHAPE, "placement needs at least 2 experts per device (E/D=%d)", G);
  auto at = [&](int i, int j) -> int64_t { return (int64_t)C_host[(size_t)i * E + j]; };
  std::vector<char> used(E, 0);
  std::vector<int> placed;   // all experts placed so far, in push order
  placed.reserve(E);
  for (int dev = 0; dev < D; ++dev) {
    int* Ld = L_host + (size_t)dev * G;
    int len = 0;
    if (dev == 0) {
      int bi = 0, bj = 1;
      for (int i = 0; i < E; ++i)
        for (int j = i + 1; j < E; ++j)
          if (at(i, j) > at(bi, bj)) { bi = i; bj = j; }
      Ld[len++] = bi; Ld[len++] = bj;
      used[bi] = used[bj] = 1;
      placed.push_back(bi); placed.push_back(bj);
    } else {
      int cand = -1;
      int64_t cand_val = 0;
      for (int e = 0; e < E; ++e) {
        if (used[e]) continue;
        int64_t v = 0;
        for (int t : placed) v += at(t, e);
        if (cand < 0 || v < cand_val) { cand = e; cand_val = v; }
      }
      Ld[len++] = cand;
      used[cand] = 1;
      placed.push_back(cand);
    }
    while (len < G) {
      int cand = -1;
      int64_t cand_val = 0;
      for (int e = 0; e < E; ++e) {
        if (used[e]) continue;
        int64_t v = 0;
        for (int i = 0; i < len; ++i) v += at(Ld[i], e);
        if (cand < 0 || v > cand_val) { cand = e; cand_val = v; }
      }
      Ld[len++] = cand;
      used[cand] = 1;
      placed.push_back(cand);
    }
  }
  for (int dev = 0; dev < D; ++dev)
    for (int sl = 0; sl < G; ++sl) expert_pos_host[L_host[(size_t)dev * G + sl]] = dev * G + sl;
  return OCCULT_OK;
}
