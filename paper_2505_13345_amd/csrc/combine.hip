// occult_combine: the two-stage aggregation of Eq. 0 (paper Sec. 3.1; App. A.2 "Weight
// Modulation", the accumulation of "SMM with Merging", and "Combine").
//
// Stage 1 is what each device does before the return trip: the outputs of a token's experts on
// that device are weighted by their gates and summed (slot order, f32) into one SFD row, which
// is stored in the layer's element type because it is the return payload.  Stage 2 is the
// source rank after the return trip: a token's SFD rows are summed in ascending device order.
//
// The printed Combine re-reads the whole SFD tensor once per device.  Here one wavefront owns
// one token and runs both stages back to back: the SFD row it has just rounded and stored is
// added to the token's accumulator from registers, so sfd_y is written once and not read again.
// Traffic per token: k EPD rows in, c_t SFD rows out, one ORI row out (+ one shared row in).
// The arithmetic (orders, roundings) is that of the two separate stages; no atomics.
//
// With unit weights the same kernel is the backward of dispatch and of the first product's row
// gather (occult_dispatch_backward): both are sums of replicas back into the row they came from.
#include "common.h"

namespace occult {

constexpr int kCombWaves = 4;

// AHEAD (needs lists_fit and a row within 64 * VPL vectors): the token's EPD rows are walked as one list in lane order
// (= device order, then slot order) and the next row is requested before the current one is summed, so a wave has
// two rows in flight instead of one (a third changed nothing).  The sums, their order and their roundings are those of the other path.
template <bool BF16, int VPL, bool AHEAD>
__global__ __launch_bounds__(kCombWaves * 64) void combine_kernel(
    const void* __restrict__ epd_y, void* __restrict__ sfd_y, const void* __restrict__ y_shared,
    void* __restrict__ y, const int32_t* __restrict__ tok_sfd_row,
    const int32_t* __restrict__ sfd_epd_rows, const float* __restrict__ epd_gate, int T, int D, int M1,
    int row_vecs, int lists_fit) {
  using R = Row<BF16>;
  constexpr int NE = R::kElems;
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kCombWaves + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * kCombWaves;
  for (int t = wave; t < T; t += nwaves) {
    // The token's index lists in three wave-wide loads instead of one dependent load per entry
    // (D <= 64 and, when lists_fit, min(k, D) * M1 <= 64): lane j reads the SFD row on device j,
    // the rows are compacted in device order, lane (o, m) reads EPD row and gate m of the o-th one.
    int n_dev = D, my_row = -1, my_q = -1;
    float my_g = 0.0f;
    if (lists_fit) {
      const int rl = lane < D ? tok_sfd_row[(size_t)t * D + lane] : -1;
      const unsigned long long present = __ballot(rl >= 0);
      n_dev = __popcll(present);
      const int ord = __popcll(present & ((1ull << lane) - 1ull));
      // push each present row to lane `ord` (absent lanes push to lane 63 + their own, dropped by the mask below)
      my_row = __builtin_amdgcn_ds_permute((rl >= 0 ? ord : 63) * 4, rl);
      if (lane >= n_dev) my_row = -1;
      const int o = lane / M1, m = lane - o * M1;
      const int r_o = __shfl(my_row, o < 64 ? o : 0, 64);
      if (o < n_dev) {
        my_q = sfd_epd_rows[(size_t)r_o * M1 + m];
        if (my_q >= 0) my_g = epd_gate ? epd_gate[my_q] : 1.0f;
      }
    }

    if constexpr (AHEAD) {
      typedef typename R::Raw Raw;
      const int my_o = lane / M1;   // lane (o, m): which of the token's devices the lane's entry belongs to
      unsigned long long todo = __ballot(my_q >= 0);
      const int n_rows = __popcll(todo);
      Raw cur[VPL], nxt[VPL];
      int e_cur = 0, e_nxt = 0;
      auto request = [&](int e, Raw (&into)[VPL]) {
        const int q = __builtin_amdgcn_readlane(my_q, e);
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          const int c = lane + 64 * v;
          if (c < row_vecs) into[v] = R::load_raw(epd_y, (size_t)q, row_vecs, c);
        }
      };
      if (n_rows > 0) {
        e_cur = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        request(e_cur, cur);
      }

      float acc[VPL][NE], part[VPL][NE];
#pragma unroll
      for (int v = 0; v < VPL; ++v)
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[v][e] = part[v][e] = 0.0f;
      for (int i = 0; i < n_rows; ++i) {
        const bool more = i + 1 < n_rows;
        if (more) {   // wave-uniform
          e_nxt = __ffsll((long long)todo) - 1;
          todo &= todo - 1;
          request(e_nxt, nxt);
        }
        const float g = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_g), e_cur));
        const int j = __builtin_amdgcn_readlane(my_o, e_cur);
        const bool last_of_device = !more || __builtin_amdgcn_readlane(my_o, e_nxt) != j;
        const int r = __builtin_amdgcn_readlane(my_row, j);
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          const int c = lane + 64 * v;
          if (c < row_vecs) {
            float x[NE];
            R::unpack(cur[v], x);
#pragma unroll
            for (int e = 0; e < NE; ++e) part[v][e] = fmaf(g, x[e], part[v][e]);
            if (last_of_device) {   // wave-uniform: the return payload, then stage 2 on the rounded values
              R::store_round(sfd_y, (size_t)r, row_vecs, c, part[v]);
#pragma unroll
              for (int e = 0; e < NE; ++e) {
                acc[v][e] += part[v][e];
                part[v][e] = 0.0f;
              }
            }
          }
        }
#pragma unroll
        for (int v = 0; v < VPL; ++v) cur[v] = nxt[v];
        e_cur = e_nxt;
      }
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        const int c = lane + 64 * v;
        if (c < row_vecs) {
          if (y_shared) {
            float sh[NE];
            R::load(y_shared, (size_t)t, row_vecs, c, sh);
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[v][e] += sh[e];
          }
          R::store_round(y, (size_t)t, row_vecs, c, acc[v]);
        }
      }
      continue;
    }
    // rows longer than 64 * VPL vectors are done in column chunks; the index lists stay in registers
    for (int cbase = 0; cbase < row_vecs; cbase += 64 * VPL) {
    float acc[VPL][NE];
#pragma unroll
    for (int i = 0; i < VPL; ++i)
#pragma unroll
      for (int e = 0; e < NE; ++e) acc[i][e] = 0.0f;
    for (int j = 0; j < n_dev; ++j) {
      int r;
      if (lists_fit) {
        r = __builtin_amdgcn_readlane(my_row, j);
      } else {
        r = tok_sfd_row[(size_t)t * D + j];   // wave-uniform
        if (r < 0) continue;
      }
      float part[VPL][NE];
#pragma unroll
      for (int i = 0; i < VPL; ++i)
#pragma unroll
        for (int e = 0; e < NE; ++e) part[i][e] = 0.0f;
      // stage 1: gate-weighted sum of this device's expert outputs, slot order
      for (int m = 0; m < M1; ++m) {
        int q;
        float g;
        if (lists_fit) {
          q = __builtin_amdgcn_readlane(my_q, j * M1 + m);
          if (q < 0) break;
          g = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_g), j * M1 + m));
        } else {
          q = sfd_epd_rows[(size_t)r * M1 + m];
          if (q < 0) break;
          g = epd_gate ? epd_gate[q] : 1.0f;
        }
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
          const int c = cbase + lane + 64 * i;
          if (c < row_vecs) {
            float v[NE];
            R::load(epd_y, (size_t)q, row_vecs, c, v);
#pragma unroll
            for (int e = 0; e < NE; ++e) part[i][e] = fmaf(g, v[e], part[i][e]);
          }
        }
      }
      // the return payload, then stage 2 on the rounded values
#pragma unroll
      for (int i = 0; i < VPL; ++i) {
        const int c = cbase + lane + 64 * i;
        if (c < row_vecs) {
          R::store_round(sfd_y, (size_t)r, row_vecs, c, part[i]);
#pragma unroll
          for (int e = 0; e < NE; ++e) acc[i][e] += part[i][e];
        }
      }
    }
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      const int c = cbase + lane + 64 * i;
      if (c < row_vecs) {
        if (y_shared) {
          float v[NE];
          R::load(y_shared, (size_t)t, row_vecs, c, v);
#pragma unroll
          for (int e = 0; e < NE; ++e) acc[i][e] += v[e];
        }
        R::store_round(y, (size_t)t, row_vecs, c, acc[i]);
      }
    }
    }   // column chunks
  }
}

// launches the two-stage sum; gates == NULL means unit weights
static int launch_combine(const occult_cfg_t& c, const occult_plan_t* plan, const float* gates, const void* epd,
                          void* sfd, const void* shared, void* out, occult_stream_t stream) {
  const size_t row_bytes = (size_t)c.d * elem_size(c);
  OCC_REQUIRE(row_bytes % 16 == 0, OCCULT_EALIGN, "row of %zu bytes is not a multiple of 16", row_bytes);
  OCC_REQUIRE(aligned16(epd) && aligned16(sfd) && aligned16(out) && aligned16(shared), OCCULT_EALIGN,
              "a buffer is not 16-byte aligned");
  const int row_vecs = (int)(row_bytes / 16);
  const int vpl = (row_vecs + 63) / 64;   // beyond 8 the kernel walks the row in chunks of 8 KiB
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid((c.T + kCombWaves - 1) / kCombWaves), block(kCombWaves * 64);
  const int M1 = merge_width(c);
  const int lists_fit = min_i(c.k, c.D) * M1 <= 64 ? 1 : 0;
  const bool ahead = lists_fit && vpl <= 8;
#define OCC_COMB(B, N)                                                                                     \
  do {                                                                                                     \
    if (ahead)                                                                                             \
      hipLaunchKernelGGL((combine_kernel<B, N, true>), grid, block, 0, s, epd, sfd, shared, out,           \
                         plan->tok_sfd_row, plan->sfd_epd_rows, gates, c.T, c.D, M1, row_vecs, lists_fit); \
    else                                                                                                   \
      hipLaunchKernelGGL((combine_kernel<B, N, false>), grid, block, 0, s, epd, sfd, shared, out,          \
                         plan->tok_sfd_row, plan->sfd_epd_rows, gates, c.T, c.D, M1, row_vecs, lists_fit); \
  } while (0)
  if (c.dtype == OCCULT_BF16) {
    if (vpl <= 1) OCC_COMB(true, 1);
    else if (vpl <= 2) OCC_COMB(true, 2);
    else if (vpl <= 4) OCC_COMB(true, 4);
    else OCC_COMB(true, 8);
  } else {
    if (vpl <= 1) OCC_COMB(false, 1);
    else if (vpl <= 2) OCC_COMB(false, 2);
    else if (vpl <= 4) OCC_COMB(false, 4);
    else OCC_COMB(false, 8);
  }
#undef OCC_COMB
  OCC_LAUNCH_CHECK("combine_kernel");
  return OCCULT_OK;
}

}  // namespace occult

using namespace occult;

extern "C" int occult_combine(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* epd_y,
                              void* sfd_y, const void* y_shared, void* y, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(plan && plan->tok_sfd_row && plan->sfd_epd_rows && plan->epd_gate, OCCULT_ENULLPTR,
              "plan or one of its tables is NULL");
  OCC_REQUIRE(epd_y && sfd_y && y, OCCULT_ENULLPTR, "epd_y, sfd_y or y is NULL");
  return launch_combine(c, plan, plan->epd_gate, epd_y, sfd_y, y_shared, y, stream);
}

// Transpose of the SFD -> EPD row gather and of dispatch: the same two-stage sum with unit weights.
extern "C" int occult_dispatch_backward(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* epd_dx,
                                        void* sfd_dx, const void* dx_shared, void* dx, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(plan && plan->tok_sfd_row && plan->sfd_epd_rows, OCCULT_ENULLPTR, "plan or one of its tables is NULL");
  OCC_REQUIRE(epd_dx && sfd_dx && dx, OCCULT_ENULLPTR, "epd_dx, sfd_dx or dx is NULL");
  return launch_combine(c, plan, nullptr, epd_dx, sfd_dx, dx_shared, dx, stream);
}
