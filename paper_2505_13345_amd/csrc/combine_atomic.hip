// occult_combine_atomic: the two-stage combine with the paper's own first stage, an atomic merge
// (paper Sec. 3.1: several thread blocks write the same SFD rows, "handled through atomic_add" on a
// float32 output tensor that is converted to the target type afterwards; App. A.2 "SMM with Merging").
//
// Opt-in and not bit-reproducible: the order in which a device's expert outputs reach an SFD row is
// whatever the hardware makes it.  occult_combine (order-fixed, no atomics, one fused kernel) is the
// default path and the faster one on this chip; this entry point exists so that the two can be measured
// side by side.
//   clear   : the first N_sfd rows of the accumulation tensor are zeroed (N_sfd read on the device)
//   merge   : one wavefront per EPD row q adds epd_gate[q] * epd_y[q] into row epd_sfd_row[q]
//             mode 0: float32 atomic adds into sfd_acc (the paper's variant)
//             mode 1: packed bf16 atomic adds (two elements per operation) straight into sfd_y
//   stage 2 : one wavefront per token: mode 0 rounds each of its SFD rows to the storage type and stores it
//             (the return payload); then, as in occult_combine, the rows are summed in ascending device
//             order (+ y_shared) in f32.
#include "common.h"

namespace occult {

constexpr int kAtomWaves = 4;
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(256) void clear_rows_kernel(u32x4* __restrict__ buf, const int32_t* __restrict__ dev_offset,
                                                         int D, int row_vecs) {
  const size_t n = (size_t)dev_offset[D] * row_vecs;   // N_sfd rows of row_vecs 16-byte vectors
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) buf[i] = z;
}

template <bool BF16, int MODE>
__global__ __launch_bounds__(kAtomWaves * 64) void merge_atomic_kernel(
    const void* __restrict__ epd_y, float* __restrict__ sfd_acc, void* __restrict__ sfd_y,
    const int32_t* __restrict__ epd_sfd_row, const float* __restrict__ epd_gate, int n_epd, int d, int row_vecs) {
  using R = Row<BF16>;
  constexpr int NE = R::kElems;
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kAtomWaves + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * kAtomWaves;
  for (int q = wave; q < n_epd; q += nwaves) {
    const int r = epd_sfd_row[q];
    const float g = epd_gate[q];
    for (int c = lane; c < row_vecs; c += 64) {
      float v[NE];
      R::load(epd_y, (size_t)q, row_vecs, c, v);
      if (MODE == 0) {
        float* dst = sfd_acc + (size_t)r * d + (size_t)c * NE;
#pragma unroll
        for (int e = 0; e < NE; ++e) unsafeAtomicAdd(dst + e, g * v[e]);
      } else {
        auto* dst = reinterpret_cast<__attribute__((address_space(1))) bf16x2_t*>(
            reinterpret_cast<uintptr_t>(static_cast<char*>(sfd_y) + ((size_t)r * row_vecs + c) * 16));
#pragma unroll
        for (int e = 0; e < NE; e += 2) {
          const bf16x2_t p = {(__bf16)(g * v[e]), (__bf16)(g * v[e + 1])};
          __builtin_amdgcn_global_atomic_fadd_v2bf16(dst + e / 2, p);
        }
      }
    }
  }
}

template <bool BF16, int MODE>
__global__ __launch_bounds__(kAtomWaves * 64) void combine_stage2_kernel(
    const float* __restrict__ sfd_acc, void* __restrict__ sfd_y, const void* __restrict__ y_shared,
    void* __restrict__ y, const int32_t* __restrict__ tok_sfd_row, int T, int D, int d, int row_vecs) {
  using R = Row<BF16>;
  constexpr int NE = R::kElems;
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kAtomWaves + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * kAtomWaves;
  for (int t = wave; t < T; t += nwaves) {
    for (int c = lane; c < row_vecs; c += 64) {
      float acc[NE];
#pragma unroll
      for (int e = 0; e < NE; ++e) acc[e] = 0.0f;
      for (int j = 0; j < D; ++j) {   // ascending device order
        const int r = tok_sfd_row[(size_t)t * D + j];
        if (r < 0) continue;
        float v[NE];
        if (MODE == 0) {
          const float* src = sfd_acc + (size_t)r * d + (size_t)c * NE;
#pragma unroll
          for (int e = 0; e < NE; ++e) v[e] = src[e];
          R::store_round(sfd_y, (size_t)r, row_vecs, c, v);   // the return payload, rounded to the storage type
        } else {
          R::load(sfd_y, (size_t)r, row_vecs, c, v);
        }
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[e] += v[e];
      }
      if (y_shared) {
        float v[NE];
        R::load(y_shared, (size_t)t, row_vecs, c, v);
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[e] += v[e];
      }
      R::store_round(y, (size_t)t, row_vecs, c, acc);
    }
  }
}

}  // namespace occult

using namespace occult;

extern "C" int occult_combine_atomic(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* epd_y,
                                     float* sfd_acc, void* sfd_y, const void* y_shared, void* y, int mode,
                                     occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  OCC_REQUIRE(mode == 0 || mode == 1, OCCULT_EINVAL, "mode=%d must be 0 (f32 atomics) or 1 (packed bf16 atomics)", mode);
  OCC_REQUIRE(mode == 0 || c.dtype == OCCULT_BF16, OCCULT_EINVAL, "mode 1 needs a bf16 layer");
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(plan && plan->tok_sfd_row && plan->epd_sfd_row && plan->epd_gate && plan->dev_offset, OCCULT_ENULLPTR,
              "plan or one of its tables is NULL");
  OCC_REQUIRE(epd_y && sfd_y && y, OCCULT_ENULLPTR, "epd_y, sfd_y or y is NULL");
  OCC_REQUIRE(mode == 1 || sfd_acc, OCCULT_ENULLPTR, "sfd_acc is NULL (mode 0 accumulates there)");
  const size_t row_bytes = (size_t)c.d * elem_size(c);
  OCC_REQUIRE(row_bytes % 16 == 0, OCCULT_EALIGN, "row of %zu bytes is not a multiple of 16", row_bytes);
  OCC_REQUIRE(aligned16(epd_y) && aligned16(sfd_y) && aligned16(y) && aligned16(y_shared) && aligned16(sfd_acc),
              OCCULT_EALIGN, "a buffer is not 16-byte aligned");
  const int row_vecs = (int)(row_bytes / 16);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n_epd = c.T * c.k;
  // accumulation tensor: f32 rows of d elements (mode 0) or the storage-type rows of sfd_y (mode 1)
  void* target = mode == 0 ? static_cast<void*>(sfd_acc) : sfd_y;
  const int target_vecs = mode == 0 ? c.d / 4 : row_vecs;
  hipLaunchKernelGGL(clear_rows_kernel, dim3(2048), dim3(256), 0, s, static_cast<u32x4*>(target), plan->dev_offset, c.D,
                     target_vecs);
  OCC_LAUNCH_CHECK("clear_rows_kernel");
  const dim3 block(kAtomWaves * 64);
  const dim3 grid_q((unsigned)min_i((n_epd + kAtomWaves - 1) / kAtomWaves, 1 << 16));
  const dim3 grid_t((unsigned)min_i((c.T + kAtomWaves - 1) / kAtomWaves, 1 << 16));
#define OCC_ATOM(B, M)                                                                                            \
  do {                                                                                                            \
    hipLaunchKernelGGL((merge_atomic_kernel<B, M>), grid_q, block, 0, s, epd_y, sfd_acc, sfd_y, plan->epd_sfd_row, \
                       plan->epd_gate, n_epd, c.d, row_vecs);                                                     \
    OCC_LAUNCH_CHECK("merge_atomic_kernel");                                                                      \
    hipLaunchKernelGGL((combine_stage2_kernel<B, M>), grid_t, block, 0, s, sfd_acc, sfd_y, y_shared, y,            \
                       plan->tok_sfd_row, c.T, c.D, c.d, row_vecs);                                               \
    OCC_LAUNCH_CHECK("combine_stage2_kernel");                                                                    \
  } while (0)
  if (c.dtype == OCCULT_BF16) {
    if (mode == 0) OCC_ATOM(true, 0);
    else OCC_ATOM(true, 1);
  } else {
    OCC_ATOM(false, 0);
  }
#undef OCC_ATOM
  return OCCULT_OK;
}
