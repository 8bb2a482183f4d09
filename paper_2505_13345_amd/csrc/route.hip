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

#include <float.h>
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

// Cross-lane steps on the VALU's data-parallel primitives (no LDS crossbar): four symmetric
// exchanges leave every lane of a 16-lane row with the row's result, two row broadcasts carry it
// into lane 63, which is read back as a wave-uniform value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i(int own, int v) {
  return __builtin_amdgcn_update_dpp(own, v, CTRL, ROW_MASK, 0xF, false);   // rows outside the mask keep `own`
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f(float own, float v) {
  return __builtin_bit_cast(float, dpp_i<CTRL, ROW_MASK>(__builtin_bit_cast(int, own), __builtin_bit_cast(int, v)));
}
constexpr int kQuadSwap1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kQuadSwap2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141;
constexpr int kRowMirror = 0x140;
constexpr int kRowBcast15 = 0x142;     // lane 15 of each row into the next row (rows 1 and 3 take it)
constexpr int kRowBcast31 = 0x143;     // lane 31 into rows 2 and 3

// (value, index) as one 64-bit key whose unsigned order is "larger value first, equal values -> lower index":
// the value's bits made monotone (negative floats inverted, positive ones offset) in the high word, the
// complemented index in the low word.  One 64-bit compare per step instead of three compares.
__device__ __forceinline__ unsigned long long argmax_key(float v, int i) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const unsigned ord = u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
  return ((unsigned long long)ord << 32) | (unsigned)(~i);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void argmax_step(unsigned long long& key) {
  const int lo = dpp_i<CTRL, ROW_MASK>((int)(unsigned)key, (int)(unsigned)key);
  const int hi = dpp_i<CTRL, ROW_MASK>((int)(unsigned)(key >> 32), (int)(unsigned)(key >> 32));
  const unsigned long long other = ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
  key = other > key ? other : key;
}

// larger value first, equal values -> lower index; result in every lane
__device__ __forceinline__ void wave_argmax(float& v, int& i) {
  unsigned long long key = argmax_key(v, i);
  argmax_step<kQuadSwap1, 0xF>(key);
  argmax_step<kQuadSwap2, 0xF>(key);
  argmax_step<kRowHalfMirror, 0xF>(key);
  argmax_step<kRowMirror, 0xF>(key);
  argmax_step<kRowBcast15, 0xA>(key);
  argmax_step<kRowBcast31, 0xC>(key);
  const unsigned ord = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(key >> 32), 63);
  i = ~__builtin_amdgcn_readlane((int)(unsigned)key, 63);
  v = __builtin_bit_cast(float, ord ^ ((ord >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f<kQuadSwap1, 0xF>(v, v);
  v += dpp_f<kQuadSwap2, 0xF>(v, v);
  v += dpp_f<kRowHalfMirror, 0xF>(v, v);
  v += dpp_f<kRowMirror, 0xF>(v, v);
  v += dpp_f<kRowBcast15, 0xA>(0.0f, v);
  v += dpp_f<kRowBcast31, 0xC>(0.0f, v);
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

constexpr int kRouteWavesPerBlock = 4;

// Routes one token on one wavefront.  `row` points at the token's E scores (global or LDS);
// s_dev[e] is the device of expert e.  Lane s < k writes slot s.
template <int EPL>  // experts per lane = ceil(E / 64)
__device__ __forceinline__ void route_one(const float* row, int lane, int E, int k, int D, const int* s_dev,
                                          int n_d, int prune_mode, int renorm, const int32_t* sim_table,
                                          int32_t* ids_t, float* w_t) {
  const float kNegInf = -INFINITY;
  float v0[EPL];   // the token's scores as read (with -0.0 folded onto +0.0)
  float v[EPL];    // working copy: taken / disallowed entries become -inf
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = lane + 64 * i;
    // NaN and -inf scores are read as the lowest finite value and +inf as the highest: every real
    // entry then stays above the -inf that marks taken and absent entries, so each round selects a
    // new index below E whatever the scores hold (ids index other tables downstream), and the
    // device sums and gates stay finite
    v0[i] = (e < E) ? fminf(fmaxf(row[e] + 0.0f, -FLT_MAX), FLT_MAX) : kNegInf;
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

  if (n_d > 0 && prune_mode == 3) {
    // Expert-similarity-based pruning: routed experts on kept devices stay in their slots; the
    // others are replaced, in slot (= descending score) order, by the first entry of their table
    // row that is on a kept device and not taken.  `taken` = one bit per expert, wave-uniform.
    unsigned long long taken[4] = {0ull, 0ull, 0ull, 0ull};
    for (int s = 0; s < k; ++s) {
      const int e = __shfl(my_id, s, 64);
      if ((kept >> s_dev[e]) & 1ull) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if ((e >> 6) == q) taken[q] |= 1ull << (e & 63);
      }
    }
    for (int s = 0; s < k; ++s) {
      const int e = __shfl(my_id, s, 64);
      if ((kept >> s_dev[e]) & 1ull) continue;   // wave-uniform
      const int32_t* trow = sim_table + (size_t)e * (E - 1);
      int found = -1;
      for (int base = 0; base < E - 1 && found < 0; base += 64) {
        const int q = base + lane;
        int c = 0;
        bool ok = false;
        if (q < E - 1) {
          c = trow[q];
          unsigned long long word = taken[0];
#pragma unroll
          for (int m = 1; m < 4; ++m)
            if ((c >> 6) == m) word = taken[m];
          ok = ((kept >> s_dev[c]) & 1ull) && !((word >> (c & 63)) & 1ull);
        }
        const unsigned long long hits = __ballot(ok);
        if (hits) found = __shfl(c, __ffsll((long long)hits) - 1, 64);
      }
      // host checks n_d * G >= k, so a free expert on a kept device always exists
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if ((found >> 6) == q) taken[q] |= 1ull << (found & 63);
      // its score sits in lane found % 64, register found / 64
      float fv = v0[0];
#pragma unroll
      for (int i = 1; i < EPL; ++i)
        if ((found >> 6) == i) fv = v0[i];
      fv = __shfl(fv, found & 63, 64);
      if (lane == s) {
        my_id = found;
        my_v = fv;
      }
    }
  } else if (n_d > 0) {
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
    ids_t[lane] = my_id;
    w_t[lane] = g;
  }
}

template <int EPL>
__global__ __launch_bounds__(kRouteWavesPerBlock * 64) void route_kernel(
    const float* __restrict__ logits, int T, int E, int k, int D, int G,
    const int32_t* __restrict__ expert_pos, int n_d, int prune_mode, int renorm,
    const int32_t* __restrict__ sim_table, int32_t* __restrict__ ids, float* __restrict__ w) {
  __shared__ int s_dev[OCCULT_MAX_E];
  if (n_d > 0) {   // uniform; only pruning asks which device an expert is on
    for (int e = threadIdx.x; e < E; e += blockDim.x)
      s_dev[e] = (expert_pos ? expert_pos[e] : e) / G;
    __syncthreads();
  }

  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * kRouteWavesPerBlock + (threadIdx.x >> 6);
  if (t >= T) return;   // whole wave leaves together; no barrier follows
  route_one<EPL>(logits + (size_t)t * E, lane, E, k, D, s_dev, n_d, prune_mode, renorm, sim_table,
                 ids + (size_t)t * k, w + (size_t)t * k);
}

// ------------------------------------------------------------------------------------------
// Router projection g(x) = x W_r^T (paper Eq. 1), bf16 inputs.
// The work is reading x once: a block takes 32 tokens, its 4 waves take a quarter of the hidden
// dimension each and multiply it with all E expert rows on v_mfma_f32_16x16x32_bf16 (operands
// loaded straight into fragment registers: 16 rows x one 64-byte sector per load; the expert
// rows come from cache).  The four partial products are added in LDS in wave order (a fixed
// order, so scores are reproducible) and written out as float32.  Routing runs as its own launch:
// one token per wave is a chain of dependent cross-lane steps, which many resident waves hide and
// eight tokens in sequence on one wave do not (measured: fused 75 us, separate 40 us at T = 2^14).
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4v __attribute__((ext_vector_type(4)));
constexpr int kRouterTokens = 32;

template <int EB>   // blocks of 16 experts, E <= 16 * EB
__global__ __launch_bounds__(256) void router_kernel(const __bf16* __restrict__ x, const __bf16* __restrict__ wr,
                                                     int T, int d, int E, float* __restrict__ logits) {
  constexpr int LSTRIDE = 16 * EB + 4;
  __shared__ __attribute__((aligned(16))) float s_lg[kRouterTokens * LSTRIDE];

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 15, c = lane >> 4;
  const int tok0 = blockIdx.x * kRouterTokens;
  const int kq = d / 4;   // host: d % 128 == 0
  // The MFMA wants lane l on row l % 16, K group l / 16; loaded that way neighbouring lanes would read rows a whole
  // row pitch apart (16 cache lines looked up per 16 lanes).  Rows are loaded with lane l on row l / 4, K group l % 4
  // (four neighbouring lanes = one 64-byte sector) and permuted into the MFMA's order before use (ds_bpermute: the
  // LDS crossbar, no LDS memory).
  const int lrow = lane >> 2;
  const size_t koff = ((size_t)wave * kq + (lane & 3) * 8) * 2;
  const int from_lane4 = (r * 4 + c) * 4;   // byte index of the lane that loaded what this lane multiplies
  auto to_mfma_order = [&](const bf16x8& v) {
    typedef int i32x4v __attribute__((ext_vector_type(4)));
    i32x4v t = __builtin_bit_cast(i32x4v, v);
#pragma unroll
    for (int e = 0; e < 4; ++e) t[e] = __builtin_amdgcn_ds_bpermute(from_lane4, t[e]);
    return __builtin_bit_cast(bf16x8, t);
  };
  const char* xp[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    const int t = min(tok0 + tb * 16 + lrow, T - 1);   // rows past the end repeat the last token; not written
    xp[tb] = reinterpret_cast<const char*>(x) + (size_t)t * d * 2 + koff;
  }
  const char* wp[EB];
#pragma unroll
  for (int eb = 0; eb < EB; ++eb) {
    const int e = min(eb * 16 + lrow, E - 1);
    wp[eb] = reinterpret_cast<const char*>(wr) + (size_t)e * d * 2 + koff;
  }
  f32x4v acc[2][EB];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int eb = 0; eb < EB; ++eb) acc[tb][eb] = f32x4v{0.0f, 0.0f, 0.0f, 0.0f};

  // K steps of 32.  The hidden rows are what comes from HBM: XS steps of them (16 rows x 64 bytes
  // each) are fetched in one go, two such chunks deep, while the expert rows (cache hits) are
  // fetched one step ahead of their use.
  constexpr int XS = EB <= 4 ? 8 : (EB == 8 ? 4 : 2);
  const int nst = kq / 32;
  struct Chunk {
    bf16x8 xf[XS][2];
  };
  auto load_x = [&](Chunk& ch, int first) {
#pragma unroll
    for (int q = 0; q < XS; ++q) {
      const int st = min(first + q, nst - 1);   // past the end the last step is fetched again and not used
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
        ch.xf[q][tb] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(xp[tb] + (size_t)st * 64));
    }
  };
  constexpr int WD = EB <= 4 ? 4 : 2;   // expert-row fragments in flight (steps ahead + 1)
  bf16x8 wf[WD][EB];
  auto load_w = [&](int buf, int st) {
    st = min(st, nst - 1);
#pragma unroll
    for (int eb = 0; eb < EB; ++eb) wf[buf][eb] = *reinterpret_cast<const bf16x8*>(wp[eb] + (size_t)st * 64);
  };
  auto multiply = [&](const Chunk& ch, int first) {
#pragma unroll
    for (int q = 0; q < XS; ++q) {
      load_w((q + WD - 1) % WD, first + q + WD - 1);
      if (first + q < nst) {
        bf16x8 xo[2], wo[EB];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) xo[tb] = to_mfma_order(ch.xf[q][tb]);
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) wo[eb] = to_mfma_order(wf[q % WD][eb]);
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
          for (int eb = 0; eb < EB; ++eb)
            acc[tb][eb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wo[eb], xo[tb], acc[tb][eb], 0, 0, 0);
      }
    }
  };
  Chunk c0, c1;
  load_x(c0, 0);
#pragma unroll
  for (int q = 0; q < WD - 1; ++q) load_w(q, q);
  for (int first = 0; first < nst; first += 2 * XS) {
    load_x(c1, first + XS);
    multiply(c0, first);
    load_x(c0, first + 2 * XS);
    multiply(c1, first + XS);
  }

  // acc[tb][eb] element j of lane l: token tb*16 + l%16, expert eb*16 + (l/16)*4 + j
#pragma unroll
  for (int turn = 0; turn < 4; ++turn) {
    if (wave == turn) {
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) {
          f32x4v* dst = reinterpret_cast<f32x4v*>(&s_lg[(tb * 16 + r) * LSTRIDE + eb * 16 + c * 4]);
          f32x4v v = acc[tb][eb];
          if (turn > 0) {
            const f32x4v old = *dst;
            v = old + v;
          }
          *dst = v;
        }
    }
    __syncthreads();
  }

  // scores out: wave w writes tokens w*8 .. w*8+7 of the block, rows of E floats
  for (int j = 0; j < kRouterTokens / 4; ++j) {
    const int tl = wave * (kRouterTokens / 4) + j;
    const int t = tok0 + tl;
    if (t >= T) break;   // wave-uniform; no barrier follows
    const float* row = &s_lg[tl * LSTRIDE];
    for (int e = lane; e < E; e += 64) logits[(size_t)t * E + e] = row[e];
  }
}

// float32 inputs (parity configuration): one thread per (token, expert), K summed in order
__global__ __launch_bounds__(256) void router_f32_kernel(const float* __restrict__ x, const float* __restrict__ wr,
                                                         int T, int d, int E, float* __restrict__ logits) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)T * E) return;
  const float* xr = x + (i / E) * d;
  const float* wrow = wr + (i % E) * d;
  float acc = 0.0f;
  for (int q = 0; q < d; ++q) acc = acc + xr[q] * wrow[q];
  logits[i] = acc;
}

// Gram matrix of router scores, H^T H in float64.  A block takes a slice of tokens and a 64 x 64
// tile of the matrix: the two 64-column panels of its tokens go through LDS, every thread keeps a
// 4 x 4 patch of sums, and the tile is added to the result with double atomics.
constexpr int kGramTokens = 64;
__global__ __launch_bounds__(256) void gram_kernel(const float* __restrict__ logits, int T, int E,
                                                   int tokens_per_block, double* __restrict__ gram) {
  __shared__ float pa[kGramTokens][65], pb[kGramTokens][65];
  const int tiles = (E + 63) / 64;
  const int ti = blockIdx.y / tiles, tj = blockIdx.y % tiles;
  const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;   // patch rows ty*4.., columns tx*4..
  double acc[4][4] = {};
  const int t_begin = blockIdx.x * tokens_per_block;
  const int t_end = min(T, t_begin + tokens_per_block);
  for (int t0 = t_begin; t0 < t_end; t0 += kGramTokens) {
    for (int i = threadIdx.x; i < kGramTokens * 64; i += 256) {
      const int tt = i / 64, c = i % 64;
      const int t = t0 + tt;
      const int ea = ti * 64 + c, eb = tj * 64 + c;
      pa[tt][c] = (t < t_end && ea < E) ? logits[(size_t)t * E + ea] : 0.0f;
      pb[tt][c] = (t < t_end && eb < E) ? logits[(size_t)t * E + eb] : 0.0f;
    }
    __syncthreads();
    for (int tt = 0; tt < kGramTokens; ++tt) {
      double a[4], b[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        a[q] = (double)pa[tt][ty * 4 + q];
        b[q] = (double)pb[tt][tx * 4 + q];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = acc[i][j] + a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int ei = ti * 64 + ty * 4 + i, ej = tj * 64 + tx * 4 + j;
      if (ei < E && ej < E) atomicAdd(&gram[(size_t)ei * E + ej], acc[i][j]);
    }
}

__global__ void fill_f64(double* p, size_t n, double v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace occult

using namespace occult;

extern "C" int occult_similarity_gram(const occult_cfg_t* cfg, const float* logits, double* gram,
                                      int accumulate, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  OCC_REQUIRE(gram, OCCULT_ENULLPTR, "gram is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t n = (size_t)c.E * c.E;
  if (!accumulate) {   // a fill kernel rather than a memset node, so the call can be captured in a graph
    hipLaunchKernelGGL(fill_f64, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, gram, n, 0.0);
    OCC_LAUNCH_CHECK("fill_f64");
  }
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(logits, OCCULT_ENULLPTR, "logits is NULL");
  const int tiles = (c.E + 63) / 64;
  int slices = (c.T + 1023) / 1024;          // about 1024 tokens per block
  if (slices < 1) slices = 1;
  const int per = ((c.T + slices - 1) / slices + kGramTokens - 1) / kGramTokens * kGramTokens;
  slices = (c.T + per - 1) / per;
  hipLaunchKernelGGL(gram_kernel, dim3(slices, tiles * tiles), dim3(256), 0, s, logits, c.T, c.E, per, gram);
  OCC_LAUNCH_CHECK("gram_kernel");
  return OCCULT_OK;
}

extern "C" int occult_similarity_table(const double* gram_host, int32_t E, int32_t* table_host) {
  OCC_REQUIRE(gram_host && table_host, OCCULT_ENULLPTR, "gram_host or table_host is NULL");
  OCC_REQUIRE(E >= 2 && E <= OCCULT_MAX_E, OCCULT_EINVAL, "E=%d outside 2..%d", E, OCCULT_MAX_E);
  for (int i = 0; i < E; ++i)
    OCC_REQUIRE(gram_host[(size_t)i * E + i] > 0.0, OCCULT_EINVAL, "gram[%d][%d] is not positive", i, i);
  double sim[OCCULT_MAX_E];
  for (int i = 0; i < E; ++i) {
    for (int j = 0; j < E; ++j) {
      // each product and the quotient rounded on its own (file-wide contraction is off)
      const double g = gram_host[(size_t)i * E + j];
      const double num = g * g;
      const double den = gram_host[(size_t)i * E + i] * gram_host[(size_t)j * E + j];
      sim[j] = num / den;
    }
    int32_t* row = table_host + (size_t)i * (E - 1);
    int n = 0;
    for (int j = 0; j < E; ++j)
      if (j != i) row[n++] = j;
    // insertion sort by (similarity descending, index ascending): stable, E <= 256
    for (int a = 1; a < n; ++a) {
      const int32_t v = row[a];
      int b = a - 1;
      while (b >= 0 && sim[row[b]] < sim[v]) {
        row[b + 1] = row[b];
        --b;
      }
      row[b + 1] = v;
    }
  }
  return OCCULT_OK;
}

extern "C" int occult_route(const occult_cfg_t* cfg, const float* logits, int32_t* ids, float* w,
                            occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(logits && ids && w, OCCULT_ENULLPTR, "logits, ids or w is NULL");
  if (c.n_d > 0 && c.prune_mode == 3)
    OCC_REQUIRE(c.sim_table != nullptr, OCCULT_ENULLPTR, "prune_mode 3 needs cfg.sim_table");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int G = c.E / c.D;
  const dim3 grid((c.T + kRouteWavesPerBlock - 1) / kRouteWavesPerBlock), block(kRouteWavesPerBlock * 64);
  const int epl = (c.E + 63) / 64;
#define OCC_ROUTE_LAUNCH(N)                                                                     \
  hipLaunchKernelGGL(route_kernel<N>, grid, block, 0, s, logits, c.T, c.E, c.k, c.D, G,         \
                     c.expert_pos, c.n_d, c.prune_mode, c.renorm, c.sim_table, ids, w)
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

extern "C" int occult_router(const occult_cfg_t* cfg, const void* x, const void* w_router, float* logits,
                             int32_t* ids, float* w, occult_stream_t stream) {
  int rc = check_cfg(cfg);
  if (rc) return rc;
  const occult_cfg_t c = *cfg;
  if (c.T == 0) return OCCULT_OK;
  OCC_REQUIRE(x && w_router && logits && ids && w, OCCULT_ENULLPTR, "x, w_router, logits, ids or w is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (c.dtype == OCCULT_F32) {
    const size_t n = (size_t)c.T * c.E;
    hipLaunchKernelGGL(router_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       static_cast<const float*>(x), static_cast<const float*>(w_router), c.T, c.d, c.E, logits);
    OCC_LAUNCH_CHECK("router_f32_kernel");
    return occult_route(cfg, logits, ids, w, stream);
  }
  OCC_REQUIRE(c.d % 128 == 0, OCCULT_ESHAPE, "bf16 router needs d to be a multiple of 128 (d=%d)", c.d);
  OCC_REQUIRE(aligned16(x) && aligned16(w_router), OCCULT_EALIGN, "x or w_router is not 16-byte aligned");
  const dim3 grid((c.T + kRouterTokens - 1) / kRouterTokens), block(256);
  const int eb = (c.E + 15) / 16;
#define OCC_ROUTER_LAUNCH(N)                                                             \
  hipLaunchKernelGGL(router_kernel<N>, grid, block, 0, s, static_cast<const __bf16*>(x), \
                     static_cast<const __bf16*>(w_router), c.T, c.d, c.E, logits)
  if (eb <= 1) OCC_ROUTER_LAUNCH(1);
  else if (eb <= 2) OCC_ROUTER_LAUNCH(2);
  else if (eb <= 4) OCC_ROUTER_LAUNCH(4);
  else if (eb <= 8) OCC_ROUTER_LAUNCH(8);
  else OCC_ROUTER_LAUNCH(16);
#undef OCC_ROUTER_LAUNCH
  OCC_LAUNCH_CHECK("router_kernel");
  return occult_route(cfg, logits, ids, w, stream);
}
