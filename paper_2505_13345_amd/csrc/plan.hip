// occult_plan: the dispatch plan for all D simulated devices at once
// (paper App. A.2 "Building BRIM_0" and "Building BRIM_1"; Sec. 2.2 replica count).
//
// The printed builders are sequential counters: BRIM_0 numbers (device, token) pairs
// device-major / token-ascending, BRIM_1 numbers (local expert, SFD row) pairs expert-major /
// row-ascending.  Both are stable ranks, so they are computed here without float atomics and in a
// fixed order:
//   pass 1  plan_count : one token per thread; per block of 256 tokens, the set of its tokens that
//                        touch each device and each placement position (bit-or into LDS), and the
//                        sets' sizes;
//   pass 2  plan_scan  : one block turns the [blocks][D+E] counts into exclusive bases
//                        (column scan over blocks, then a scan over devices / positions);
//   pass 3  plan_fill  : every block rebuilds its sets; a token's rank in a column is the block's
//                        base plus the number of set bits below its own, and every token writes
//                        its own entries of the rank-addressed tables.
// Ranks are token-ascending, which is the order the sequential counters would visit: every table
// is bit-reproducible.  A batch of one block (T <= 256) runs the three passes in one launch.
#include "common.h"

#include <mutex>

namespace occult {

constexpr int kTPB = kPlanTokensPerBlock;   // 256 threads = 4 waves, one token per thread
constexpr int kMaxCols = OCCULT_MAX_D + OCCULT_MAX_E;

// Per block of 256 tokens every column (device j: column j; placement position P: column D + P) gets a 256-bit set
// of the block's tokens that touch it, built in LDS with bit-or (order-free, so deterministic).  A column's count is
// the number of set bits, a token's rank inside its block the number of set bits below its own: the same
// token-ascending ranks the sequential counters give, without a wave vote per column.
typedef unsigned long long TokenSet[4];

__device__ __forceinline__ int bits_below(const unsigned long long* col, int tl) {
  const int tw = tl >> 6;
  const unsigned long long part = (1ull << (tl & 63)) - 1ull;
  int n = 0;
#pragma unroll
  for (int wd = 0; wd < 4; ++wd) n += __popcll(col[wd] & (wd < tw ? ~0ull : (wd == tw ? part : 0ull)));
  return n;
}

// A token's selected placement positions (a position named by several slots counts once, with the gate of the
// last), their devices and gates; -1 / 0 in unused slots.  k <= KMAX.
template <int KMAX>
struct TokenSlots {
  int pos[KMAX], dev[KMAX];
  float gate[KMAX];
  unsigned long long devmask;
};

template <int KMAX, bool GATES>
__device__ __forceinline__ void load_token(TokenSlots<KMAX>& ts, const int32_t* __restrict__ ids,
                                           const float* __restrict__ w, int t, int T, int k, int G, const int* s_pos) {
#pragma unroll
  for (int s = 0; s < KMAX; ++s) {
    const bool live = (t < T) && (s < k);
    ts.pos[s] = live ? s_pos[ids[(size_t)t * k + s]] : -1;
    ts.gate[s] = (GATES && live) ? w[(size_t)t * k + s] : 0.0f;
  }
#pragma unroll
  for (int s = 0; s < KMAX; ++s)
#pragma unroll
    for (int s2 = s + 1; s2 < KMAX; ++s2)
      if (ts.pos[s] >= 0 && ts.pos[s2] == ts.pos[s]) ts.pos[s] = -1;
  ts.devmask = 0;
#pragma unroll
  for (int s = 0; s < KMAX; ++s) {
    ts.dev[s] = ts.pos[s] >= 0 ? ts.pos[s] / G : -1;
    if (ts.pos[s] >= 0) ts.devmask |= 1ull << ts.dev[s];
  }
}

// the token at bit tl of its block joins the sets of its devices and positions
template <int KMAX>
__device__ __forceinline__ void join_sets(TokenSet* s_set, int D, int tl, const TokenSlots<KMAX>& ts) {
  const unsigned long long mybit = 1ull << (tl & 63);
#pragma unroll
  for (int s = 0; s < KMAX; ++s)
    if (ts.pos[s] >= 0) {
      atomicOr(&s_set[D + ts.pos[s]][tl >> 6], mybit);
      atomicOr(&s_set[ts.dev[s]][tl >> 6], mybit);
    }
}

// Token t (bit tl of its block) writes its own entries of every table: base[c] = rank of its block's first token in
// column c.  The merge list of an SFD row is position-ascending.
template <int KMAX>
__device__ __forceinline__ void fill_token(const TokenSlots<KMAX>& ts, int t, int tl, int D, int M1, const TokenSet* s_set,
                                           const int* base, int32_t* __restrict__ tok_sfd_row,
                                           int32_t* __restrict__ sfd_token, int32_t* __restrict__ epd_sfd_row,
                                           float* __restrict__ epd_gate, int32_t* __restrict__ sfd_epd_rows) {
  for (int j = 0; j < D; ++j) {
    const bool on = (ts.devmask >> j) & 1ull;
    const int r = on ? base[j] + bits_below(s_set[j], tl) : -1;
    tok_sfd_row[(size_t)t * D + j] = r;
    if (on) {
      sfd_token[r] = t;
      int filled = 0;
#pragma unroll
      for (int s = 0; s < KMAX; ++s) filled += ts.dev[s] == j ? 1 : 0;
      for (int i = filled; i < M1; ++i) sfd_epd_rows[(size_t)r * M1 + i] = -1;
    }
  }
#pragma unroll
  for (int s = 0; s < KMAX; ++s) {
    const int P = ts.pos[s];
    if (P < 0) continue;
    const int j = ts.dev[s];
    const int r = base[j] + bits_below(s_set[j], tl);
    const int q = base[D + P] + bits_below(s_set[D + P], tl);
    int before = 0;   // this token's other positions on the same device below P
#pragma unroll
    for (int s2 = 0; s2 < KMAX; ++s2) before += (ts.dev[s2] == j && ts.pos[s2] < P) ? 1 : 0;
    epd_sfd_row[q] = r;
    epd_gate[q] = ts.gate[s];
    sfd_epd_rows[(size_t)r * M1 + before] = q;
  }
}

// pass 1: per block of 256 tokens, how many of them touch each device and each placement position
template <int KMAX>
__global__ __launch_bounds__(kTPB) void plan_count(const int32_t* __restrict__ ids, int T, int k, int E, int D, int G,
                                                   const int32_t* __restrict__ expert_pos,
                                                   uint64_t* __restrict__ tok_devmask, int32_t* __restrict__ blk_cnt) {
  static_assert(kTPB == 256, "token sets are four 64-bit words");
  __shared__ int s_pos[OCCULT_MAX_E];
  __shared__ TokenSet s_set[kMaxCols];
  const int tl = threadIdx.x, t = blockIdx.x * kTPB + tl, C = D + E;
  for (int e = tl; e < E; e += kTPB) s_pos[e] = expert_pos ? expert_pos[e] : e;
  for (int i = tl; i < C * 4; i += kTPB) (&s_set[0][0])[i] = 0ull;
  __syncthreads();
  TokenSlots<KMAX> ts;
  load_token<KMAX, false>(ts, ids, nullptr, t, T, k, G, s_pos);
  join_sets<KMAX>(s_set, D, tl, ts);
  if (t < T) tok_devmask[t] = ts.devmask;
  __syncthreads();
  for (int c = tl; c < C; c += kTPB)
    blk_cnt[(size_t)blockIdx.x * C + c] =
        __popcll(s_set[c][0]) + __popcll(s_set[c][1]) + __popcll(s_set[c][2]) + __popcll(s_set[c][3]);
}

// One block of 1024 threads.  Thread (part, c) owns rows [part*rpp, (part+1)*rpp) of column c.
constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void plan_scan(
    int32_t* __restrict__ blk_cnt, int nblk, int T, int k, int E, int D, int G,
    const int32_t* __restrict__ expert_pos, int32_t* __restrict__ dev_count,
    int32_t* __restrict__ dev_offset, int32_t* __restrict__ exp_count, int32_t* __restrict__ exp_offset,
    int32_t* __restrict__ pos_expert, uint64_t* __restrict__ counters) {
  __shared__ int s_part[kScanThreads];       // [parts][C] partial column sums
  __shared__ int s_total[kMaxCols];          // column totals
  __shared__ int s_start[kMaxCols + 2];      // exclusive scans: devices, then positions
  const int C = D + E;
  const int parts = kScanThreads / C;        // >= 3 since C <= 320
  const int rpp = (nblk + parts - 1) / parts;
  const int part = threadIdx.x / C, c = threadIdx.x % C;
  const bool active = part < parts;
  const int r0 = part * rpp, r1 = min(nblk, r0 + rpp);

  int sum = 0;
  if (active)
    for (int r = r0; r < r1; ++r) sum += blk_cnt[(size_t)r * C + c];
  if (active) s_part[part * C + c] = sum;
  __syncthreads();

  int base = 0;   // sum of this column over the parts before mine
  if (active)
    for (int p = 0; p < part; ++p) base += s_part[p * C + c];
  if (threadIdx.x < C) {
    int tot = 0;
    for (int p = 0; p < parts; ++p) tot += s_part[p * C + threadIdx.x];
    s_total[threadIdx.x] = tot;
  }
  __syncthreads();

  // exclusive scans over devices and over positions (<= 64 + 256 entries): one thread each
  if (threadIdx.x == 0) {
    int run = 0, mx = 0;
    for (int j = 0; j < D; ++j) {
      s_start[j] = run;
      dev_count[j] = s_total[j];
      dev_offset[j] = run;
      mx = max(mx, s_total[j]);
      run += s_total[j];
    }
    dev_offset[D] = run;
    counters[0] = (uint64_t)run;
    counters[3] = (uint64_t)mx;
  } else if (threadIdx.x == 64) {
    int run = 0, mx = 0;
    for (int P = 0; P < E; ++P) {
      s_start[D + P] = run;
      exp_count[P] = s_total[D + P];
      exp_offset[P] = run;
      mx = max(mx, s_total[D + P]);
      run += s_total[D + P];
    }
    exp_offset[E] = run;
    counters[1] = (uint64_t)run;
    counters[2] = (uint64_t)T * (uint64_t)k;
    counters[4] = (uint64_t)mx;
    counters[5] = counters[6] = counters[7] = 0;
  } else if (threadIdx.x >= 128 && threadIdx.x < 128 + E) {
    const int e = threadIdx.x - 128;
    pos_expert[expert_pos ? expert_pos[e] : e] = e;
  }
  // E can exceed the 896 threads after 128 only if E > 896: not possible (E <= 256)
  __syncthreads();

  if (active) {
    int run = s_start[c] + base;
    for (int r = r0; r < r1; ++r) {
      const int v = blk_cnt[(size_t)r * C + c];
      blk_cnt[(size_t)r * C + c] = run;   // count -> first rank of this block in this column
      run += v;
    }
  }
}

// pass 3: every block rebuilds its token sets and its tokens write the rank-addressed tables; blk_base holds, per
// block and column, the rank of the block's first token (pass 2)
template <int KMAX>
__global__ __launch_bounds__(kTPB) void plan_fill(
    const int32_t* __restrict__ ids, const float* __restrict__ w, int T, int k, int E, int D, int G,
    int M1, const int32_t* __restrict__ expert_pos, const int32_t* __restrict__ blk_base,
    int32_t* __restrict__ tok_sfd_row, int32_t* __restrict__ sfd_token,
    int32_t* __restrict__ epd_sfd_row, float* __restrict__ epd_gate,
    int32_t* __restrict__ sfd_epd_rows) {
  __shared__ int s_pos[OCCULT_MAX_E];
  __shared__ TokenSet s_set[kMaxCols];
  __shared__ int s_base[kMaxCols];
  const int tl = threadIdx.x, t = blockIdx.x * kTPB + tl, C = D + E;
  for (int e = tl; e < E; e += kTPB) s_pos[e] = expert_pos ? expert_pos[e] : e;
  for (int i = tl; i < C * 4; i += kTPB) (&s_set[0][0])[i] = 0ull;
  for (int c = tl; c < C; c += kTPB) s_base[c] = blk_base[(size_t)blockIdx.x * C + c];
  __syncthreads();
  TokenSlots<KMAX> ts;
  load_token<KMAX, true>(ts, ids, w, t, T, k, G, s_pos);
  join_sets<KMAX>(s_set, D, tl, ts);
  __syncthreads();
  if (t < T) fill_token<KMAX>(ts, t, tl, D, M1, s_set, s_base, tok_sfd_row, sfd_token, epd_sfd_row, epd_gate, sfd_epd_rows);
}

// A batch of at most one block of tokens (T <= 256: decode steps): the three passes in one launch of one block,
// the column counts and their scans held in LDS.  Tables bit-identical to the three-kernel path.
template <int KMAX>
__global__ __launch_bounds__(kTPB) void plan_single(
    const int32_t* __restrict__ ids, const float* __restrict__ w, int T, int k, int E, int D, int G, int M1,
    const int32_t* __restrict__ expert_pos, uint64_t* __restrict__ tok_devmask, int32_t* __restrict__ dev_count,
    int32_t* __restrict__ dev_offset, int32_t* __restrict__ exp_count, int32_t* __restrict__ exp_offset,
    int32_t* __restrict__ pos_expert, uint64_t* __restrict__ counters, int32_t* __restrict__ tok_sfd_row,
    int32_t* __restrict__ sfd_token, int32_t* __restrict__ epd_sfd_row, float* __restrict__ epd_gate,
    int32_t* __restrict__ sfd_epd_rows) {
  __shared__ int s_pos[OCCULT_MAX_E];
  __shared__ TokenSet s_set[kMaxCols];
  __shared__ int s_n[kMaxCols];       // column counts
  __shared__ int s_start[kMaxCols];   // exclusive scans: devices, then positions
  const int t = threadIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int C = D + E;
  for (int e = t; e < E; e += kTPB) s_pos[e] = expert_pos ? expert_pos[e] : e;
  for (int i = t; i < C * 4; i += kTPB) (&s_set[0][0])[i] = 0ull;
  __syncthreads();
  TokenSlots<KMAX> ts;
  load_token<KMAX, true>(ts, ids, w, t, T, k, G, s_pos);
  join_sets<KMAX>(s_set, D, t, ts);
  if (t < T) tok_devmask[t] = ts.devmask;
  __syncthreads();

  for (int c = t; c < C; c += kTPB)
    s_n[c] = __popcll(s_set[c][0]) + __popcll(s_set[c][1]) + __popcll(s_set[c][2]) + __popcll(s_set[c][3]);
  __syncthreads();

  // wave 0: devices; wave 1: positions (64 at a time, carrying the running total); waves 2, 3: inverse placement
  if (wave < 2) {
    const int n_cols = wave == 0 ? D : E, col0 = wave == 0 ? 0 : D;
    int32_t* cnt_out = wave == 0 ? dev_count : exp_count;
    int32_t* off_out = wave == 0 ? dev_offset : exp_offset;
    int run = 0, mx = 0;
    for (int c0 = 0; c0 < n_cols; c0 += 64) {
      const int c = c0 + lane;
      const int n = c < n_cols ? s_n[col0 + c] : 0;
      int incl = n;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
      }
      if (c < n_cols) {
        s_start[col0 + c] = run + incl - n;
        cnt_out[c] = n;
        off_out[c] = run + incl - n;
      }
      int m = n;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) m = max(m, __shfl_xor(m, o, 64));
      mx = max(mx, m);
      run += __shfl(incl, 63, 64);
    }
    if (lane == 0) {
      off_out[n_cols] = run;
      if (wave == 0) {
        counters[0] = (uint64_t)run;
        counters[3] = (uint64_t)mx;
      } else {
        counters[1] = (uint64_t)run;
        counters[2] = (uint64_t)T * (uint64_t)k;
        counters[4] = (uint64_t)mx;
        counters[5] = counters[6] = counters[7] = 0;
      }
    }
  } else {
    for (int e = t - 128; e < E; e += kTPB - 128) pos_expert[s_pos[e]] = e;
  }
  __syncthreads();
  if (t < T) fill_token<KMAX>(ts, t, t, D, M1, s_set, s_start, tok_sfd_row, sfd_token, epd_sfd_row, epd_gate, sfd_epd_rows);
}

size_t plan_workspace_bytes(const occult_cfg_t& c);

// The three launches of the planner on a block-count buffer `blk` of >= nblk * (D + E) ints.  plan_count
// writes every entry of the first nblk rows before plan_scan reads them: the buffer need not be cleared.
static int launch_plan(const occult_cfg_t& c, const int32_t* ids, const float* w, const occult_plan_t& p,
                       int32_t* blk, hipStream_t s) {
  const int G = c.E / c.D;
  const int nblk = (c.T + kTPB - 1) / kTPB;
  if (nblk == 1) {   // one block of tokens: the three passes in one launch (blk stays unused)
#define OCC_PLAN_SINGLE(KM)                                                                                     \
  hipLaunchKernelGGL(plan_single<KM>, dim3(1), dim3(kTPB), 0, s, ids, w, c.T, c.k, c.E, c.D, G, merge_width(c),  \
                     c.expert_pos, p.tok_devmask, p.dev_count, p.dev_offset, p.exp_count, p.exp_offset,          \
                     p.pos_expert, p.counters, p.tok_sfd_row, p.sfd_token, p.epd_sfd_row, p.epd_gate,            \
                     p.sfd_epd_rows)
    if (c.k <= 8) OCC_PLAN_SINGLE(8);
    else if (c.k <= 16) OCC_PLAN_SINGLE(16);
    else OCC_PLAN_SINGLE(32);
#undef OCC_PLAN_SINGLE
    OCC_LAUNCH_CHECK("plan_single");
    return OCCULT_OK;
  }
  if (nblk > 0) {
#define OCC_PLAN_COUNT(KM)                                                                               \
  hipLaunchKernelGGL(plan_count<KM>, dim3(nblk), dim3(kTPB), 0, s, ids, c.T, c.k, c.E, c.D, G, c.expert_pos, \
                     p.tok_devmask, blk)
    if (c.k <= 8) OCC_PLAN_COUNT(8);
    else if (c.k <= 16) OCC_PLAN_COUNT(16);
    else OCC_PLAN_COUNT(32);
#undef OCC_PLAN_COUNT
    OCC_LAUNCH_CHECK("plan_count");
  }
  // with T == 0 the scan still writes zero counts and offsets
  hipLaunchKernelGGL(plan_scan, dim3(1), dim3(kScanThreads), 0, s, blk, nblk, c.T, c.k, c.E, c.D, G,
                     c.expert_pos, p.dev_count, p.dev_offset, p.exp_count, p.exp_offset, p.pos_expert,
                     p.counters);
  OCC_LAUNCH_CHECK("plan_scan");
  if (nblk > 0) {
#define OCC_PLAN_FILL(KM)                                                                              \
  hipLaunchKernelGGL(plan_fill<KM>, dim3(nblk), dim3(kTPB), 0, s, ids, w, c.T, c.k, c.E, c.D, G,         \
                     merge_width(c), c.expert_pos, blk, p.tok_sfd_row, p.sfd_token, p.epd_sfd_row,       \
                     p.epd_gate, p.sfd_epd_rows)
    if (c.k <= 8) OCC_PLAN_FILL(8);
    else if (c.k <= 16) OCC_PLAN_FILL(16);
    else OCC_PLAN_FILL(32);
#undef OCC_PLAN_FILL
    OCC_LAUNCH_CHECK("plan_fill");
  }
  return OCCULT_OK;
}

static int check_plan_args(const occult_cfg_t& c, const int32_t* ids, const float* w, const occult_plan_t* plan) {
  OCC_REQUIRE(plan, OCCULT_ENULLPTR, "plan is NULL");
  const occult_plan_t& p = *plan;
  OCC_REQUIRE(p.tok_devmask && p.dev_count && p.dev_offset && p.tok_sfd_row && p.sfd_token &&
                  p.exp_count && p.exp_offset && p.pos_expert && p.epd_sfd_row && p.epd_gate &&
                  p.sfd_epd_rows && p.counters,
              OCCULT_ENULLPTR, "a plan table is NULL (use occult_plan_bind)");
  OCC_REQUIRE(c.T == 0 || (ids && w), OCCULT_ENULLPTR, "ids or w is NULL");
  return OCCULT_OK;
}

// Scratch of occult_plan_static: the planner's per-block counts in a device array of the library
// itself (4 MiB on every GPU the library runs on, held until the process ends).  On the host this
// name only stands for the array: its device address comes from hipGetSymbolAddress, once per
// device, and is what the kernels receive.
constexpr size_t kStaticPlanInts = (size_t)OCCULT_PLAN_STATIC_MAX_BYTES / sizeof(int32_t);
static __device__ __align__(256) int32_t scratch[kStaticPlanInts];

constexpr int kMaxHipDevices = 64;
static std::mutex g_scratch_mutex;
static int32_t* g_scratch_ptr[kMaxHipDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call for that device).
static int static_scratch(int32_t** out) {
  int dev = -1;
  OCC_HIP(hipGetDevice(&dev));
  OCC_REQUIRE(dev >= 0 && dev < kMaxHipDevices, OCCULT_EINVAL, "HIP device %d outside 0..%d", dev, kMaxHipDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    OCC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    OCC_REQUIRE(ptr, OCCULT_EHIP, "hipGetSymbolAddress returned a NULL address for the planner's scratch");
    g_scratch_ptr[dev] = static_cast<int32_t*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return OCCULT_OK;
}

}  // namespace occult

using namespace occult;

extern "C" int occult_plan(const occult_cfg_t* cfg, const int32_t* ids, const float* w,
                           const occult_plan_t* plan, void* ws, size_t ws_bytes, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  rc = check_plan_args(c, ids, w, plan);
  if (rc) return rc;
  OCC_REQUIRE(ws, OCCULT_ENULLPTR, "workspace is NULL");
  OCC_REQUIRE(ws_bytes >= plan_workspace_bytes(c), OCCULT_EWORKSPACE, "workspace of %zu bytes < required %zu",
              ws_bytes, plan_workspace_bytes(c));
  return launch_plan(c, ids, w, *plan, static_cast<int32_t*>(ws), static_cast<hipStream_t>(stream));
}

extern "C" int occult_plan_static(const occult_cfg_t* cfg, const int32_t* ids, const float* w,
                                  const occult_plan_t* plan, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  const size_t need = plan_workspace_bytes(c);
  OCC_REQUIRE(need <= (size_t)OCCULT_PLAN_STATIC_MAX_BYTES, OCCULT_EWORKSPACE,
              "this layer's planner scratch (%zu bytes for T=%d, D+E=%d) exceeds the %zu bytes of the built-in "
              "buffer: use occult_plan with a caller workspace",
              need, c.T, c.D + c.E, (size_t)OCCULT_PLAN_STATIC_MAX_BYTES);
  rc = check_plan_args(c, ids, w, plan);
  if (rc) return rc;
  int32_t* blk = nullptr;
  rc = static_scratch(&blk);
  if (rc) return rc;
  return launch_plan(c, ids, w, *plan, blk, static_cast<hipStream_t>(stream));
}
