// Host-side pieces of the C ABI that launch nothing: version, error text, argument checks,
// plan memory layout, plan statistics.
#include "common.h"

#include <string.h>

namespace occult {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int check_cfg(const occult_cfg_t* cfg) {
  OCC_REQUIRE(cfg != nullptr, OCCULT_ENULLPTR, "cfg is NULL");
  const occult_cfg_t& c = *cfg;
  OCC_REQUIRE(c.T >= 0, OCCULT_EINVAL, "T=%d must be >= 0", c.T);
  OCC_REQUIRE(c.E >= 1 && c.E <= OCCULT_MAX_E, OCCULT_EINVAL, "E=%d outside 1..%d", c.E, OCCULT_MAX_E);
  OCC_REQUIRE(c.D >= 1 && c.D <= OCCULT_MAX_D, OCCULT_EINVAL, "D=%d outside 1..%d", c.D, OCCULT_MAX_D);
  OCC_REQUIRE(c.E % c.D == 0, OCCULT_ESHAPE, "E=%d is not divisible by D=%d", c.E, c.D);
  OCC_REQUIRE(c.k >= 1 && c.k <= c.E && c.k <= OCCULT_MAX_K, OCCULT_EINVAL,
              "k=%d outside 1..min(E=%d, %d)", c.k, c.E, OCCULT_MAX_K);
  OCC_REQUIRE((int64_t)c.T * c.k < (int64_t)INT32_MAX, OCCULT_EINVAL, "T*k overflows int32");
  OCC_REQUIRE(c.S >= 0 && c.S <= 64, OCCULT_EINVAL, "S=%d outside 0..64", c.S);
  OCC_REQUIRE((int64_t)c.T * c.S < (int64_t)INT32_MAX, OCCULT_EINVAL, "T*S overflows int32");
  OCC_REQUIRE(c.d >= 1 && c.f >= 1, OCCULT_EINVAL, "d=%d, f=%d must be positive", c.d, c.f);
  OCC_REQUIRE(c.dtype == OCCULT_F32 || c.dtype == OCCULT_BF16, OCCULT_EINVAL, "unknown dtype %d", c.dtype);
  OCC_REQUIRE(c.n_d >= 0 && c.n_d <= c.D, OCCULT_EINVAL, "n_d=%d outside 0..D=%d", c.n_d, c.D);
  if (c.n_d > 0) {
    OCC_REQUIRE(c.prune_mode >= 1 && c.prune_mode <= 3, OCCULT_EINVAL, "prune_mode=%d must be 1, 2 or 3",
                c.prune_mode);
    OCC_REQUIRE((int64_t)c.n_d * (c.E / c.D) >= c.k, OCCULT_ESHAPE,
                "n_d=%d devices of %d experts cannot hold k=%d experts", c.n_d, c.E / c.D, c.k);
  }
  OCC_REQUIRE(c.renorm == 0 || c.renorm == 1, OCCULT_EINVAL, "renorm=%d must be 0 or 1", c.renorm);
  OCC_REQUIRE(c.ffn_phase >= 0 && c.ffn_phase <= 2, OCCULT_EINVAL, "ffn_phase=%d must be 0, 1 or 2", c.ffn_phase);
  return OCCULT_OK;
}

// Plan block layout: every table starts 256-byte aligned, in the order of occult_plan_t.
struct PlanLayout {
  size_t off[12];
  size_t total;
};

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

static PlanLayout plan_layout(const occult_cfg_t& c) {
  PlanLayout L;
  size_t T = (size_t)c.T, D = (size_t)c.D, E = (size_t)c.E, k = (size_t)c.k;
  size_t nsfd = (size_t)sfd_rows_max(c), m1 = (size_t)merge_width(c);
  size_t sizes[12] = {
      T * 8,              // tok_devmask
      D * 4,              // dev_count
      (D + 1) * 4,        // dev_offset
      T * D * 4,          // tok_sfd_row
      nsfd * 4,           // sfd_token
      E * 4,              // exp_count
      (E + 1) * 4,        // exp_offset
      E * 4,              // pos_expert
      T * k * 4,          // epd_sfd_row
      T * k * 4,          // epd_gate
      nsfd * m1 * 4,      // sfd_epd_rows
      8 * 8,              // counters
  };
  size_t o = 0;
  for (int i = 0; i < 12; ++i) {
    L.off[i] = o;
    o += align256(sizes[i] ? sizes[i] : 1);
  }
  L.total = o;
  return L;
}

size_t plan_workspace_bytes(const occult_cfg_t& c) {
  size_t nblk = ((size_t)c.T + kPlanTokensPerBlock - 1) / kPlanTokensPerBlock;
  if (nblk == 0) nblk = 1;
  return align256(nblk * (size_t)(c.D + c.E) * 4);
}

}  // namespace occult

using namespace occult;

extern "C" int occult_version(void) { return OCCULT_VERSION; }

extern "C" const char* occult_last_error(void) { return g_err; }

extern "C" int occult_plan_sizes(const occult_cfg_t* cfg, size_t* plan_bytes, size_t* workspace_bytes) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  OCC_REQUIRE(plan_bytes && workspace_bytes, OCCULT_ENULLPTR, "output pointer is NULL");
  *plan_bytes = plan_layout(*cfg).total;
  *workspace_bytes = plan_workspace_bytes(*cfg);
  return OCCULT_OK;
}

extern "C" int occult_plan_bind(const occult_cfg_t* cfg, void* plan_mem, size_t plan_bytes,
                                occult_plan_t* out) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  OCC_REQUIRE(plan_mem && out, OCCULT_ENULLPTR, "plan_mem or out is NULL");
  OCC_REQUIRE(((uintptr_t)plan_mem & 255u) == 0, OCCULT_EALIGN, "plan_mem is not 256-byte aligned");
  PlanLayout L = plan_layout(*cfg);
  OCC_REQUIRE(plan_bytes >= L.total, OCCULT_EWORKSPACE, "plan block of %zu bytes < required %zu",
              plan_bytes, L.total);
  char* b = static_cast<char*>(plan_mem);
  out->tok_devmask = reinterpret_cast<uint64_t*>(b + L.off[0]);
  out->dev_count = reinterpret_cast<int32_t*>(b + L.off[1]);
  out->dev_offset = reinterpret_cast<int32_t*>(b + L.off[2]);
  out->tok_sfd_row = reinterpret_cast<int32_t*>(b + L.off[3]);
  out->sfd_token = reinterpret_cast<int32_t*>(b + L.off[4]);
  out->exp_count = reinterpret_cast<int32_t*>(b + L.off[5]);
  out->exp_offset = reinterpret_cast<int32_t*>(b + L.off[6]);
  out->pos_expert = reinterpret_cast<int32_t*>(b + L.off[7]);
  out->epd_sfd_row = reinterpret_cast<int32_t*>(b + L.off[8]);
  out->epd_gate = reinterpret_cast<float*>(b + L.off[9]);
  out->sfd_epd_rows = reinterpret_cast<int32_t*>(b + L.off[10]);
  out->counters = reinterpret_cast<uint64_t*>(b + L.off[11]);
  return OCCULT_OK;
}

extern "C" int occult_plan_stats(const occult_cfg_t* cfg, const occult_plan_t* plan,
                                 occult_stats_t* out_host, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  OCC_REQUIRE(plan && out_host, OCCULT_ENULLPTR, "plan or out_host is NULL");
  OCC_REQUIRE(plan->counters, OCCULT_ENULLPTR, "plan->counters is NULL");
  uint64_t h[8];
  hipStream_t s = static_cast<hipStream_t>(stream);
  OCC_HIP(hipMemcpyAsync(h, plan->counters, sizeof(h), hipMemcpyDeviceToHost, s));
  OCC_HIP(hipStreamSynchronize(s));
  const uint64_t row = (uint64_t)cfg->d * (uint64_t)elem_size(*cfg);
  out_host->n_sfd = h[0];
  out_host->n_epd = h[1];
  out_host->rows_std = h[2];
  out_host->max_dev_count = h[3];
  out_host->max_exp_count = h[4];
  out_host->bytes_occ = 2 * h[0] * row;
  out_host->bytes_std = 2 * h[2] * row;
  out_host->bytes_meta = h[0] * (uint64_t)cfg->k * 8;
  out_host->c_t = cfg->T > 0 ? (double)h[0] / (double)cfg->T : 0.0;
  return OCCULT_OK;
}
