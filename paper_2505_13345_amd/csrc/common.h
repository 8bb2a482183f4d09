// Internal helpers shared by the library's translation units (host-side checks, error text,
// small device utilities).  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "../../include/occult.h"

namespace occult {

void set_error(const char* fmt, ...);

#define OCC_FAIL(code, ...)            \
  do {                                 \
    ::occult::set_error(__VA_ARGS__);  \
    return (code);                     \
  } while (0)

#define OCC_REQUIRE(cond, code, ...)   \
  do {                                 \
    if (!(cond)) OCC_FAIL(code, __VA_ARGS__); \
  } while (0)

#define OCC_HIP(expr)                                                              \
  do {                                                                             \
    hipError_t _e = (expr);                                                        \
    if (_e != hipSuccess)                                                          \
      OCC_FAIL(OCCULT_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e));        \
  } while (0)

// after a kernel launch: report launch-time errors without synchronising
#define OCC_LAUNCH_CHECK(name)                                                     \
  do {                                                                             \
    hipError_t _e = hipGetLastError();                                             \
    if (_e != hipSuccess)                                                          \
      OCC_FAIL(OCCULT_EHIP, "launch of %s failed: %s", name, hipGetErrorString(_e)); \
  } while (0)

// Validates the fields every call depends on. Returns OCCULT_OK or an error code (message set).
int check_cfg(const occult_cfg_t* cfg);

inline int elem_size(const occult_cfg_t& c) { return c.dtype == OCCULT_BF16 ? 2 : 4; }
inline int min_i(int a, int b) { return a < b ? a : b; }
inline int sfd_rows_max(const occult_cfg_t& c) { return c.T * min_i(c.k, c.D); }
inline int merge_width(const occult_cfg_t& c) { return min_i(c.k, c.E / c.D); }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t plan_workspace_bytes(const occult_cfg_t& c);

// native 16-byte vectors (usable with the nontemporal builtins)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(unsigned u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(unsigned u) { return __uint_as_float(u & 0xFFFF0000u); }
// two floats -> two bf16 (round to nearest even) packed low | high << 16
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));   // one packed conversion
}

// One 16-byte vector of a hidden row as floats: load, and store with the rounding of the storage type.
template <bool BF16>
struct Row;

// bf16: a 16-byte vector = 8 elements
template <>
struct Row<true> {
  static constexpr int kElems = 8;
  typedef u32x4 Raw;   // a vector as loaded
  __device__ static Raw load_raw(const void* base, size_t row, int row_vecs, int c) {
    return __builtin_nontemporal_load(static_cast<const u32x4*>(base) + row * row_vecs + c);
  }
  __device__ static void unpack(const Raw& v, float* out) {
    out[0] = bf16_lo(v.x); out[1] = bf16_hi(v.x);
    out[2] = bf16_lo(v.y); out[3] = bf16_hi(v.y);
    out[4] = bf16_lo(v.z); out[5] = bf16_hi(v.z);
    out[6] = bf16_lo(v.w); out[7] = bf16_hi(v.w);
  }
  __device__ static void load(const void* base, size_t row, int row_vecs, int c, float* out) {
    unpack(load_raw(base, row, row_vecs, c), out);
  }
  // stores the rounded values and returns them in `vals`
  __device__ static void store_round(void* base, size_t row, int row_vecs, int c, float* vals) {
    u32x4 v;
    v.x = pack_bf16(vals[0], vals[1]);
    v.y = pack_bf16(vals[2], vals[3]);
    v.z = pack_bf16(vals[4], vals[5]);
    v.w = pack_bf16(vals[6], vals[7]);
    __builtin_nontemporal_store(v, static_cast<u32x4*>(base) + row * row_vecs + c);
    vals[0] = bf16_lo(v.x); vals[1] = bf16_hi(v.x);
    vals[2] = bf16_lo(v.y); vals[3] = bf16_hi(v.y);
    vals[4] = bf16_lo(v.z); vals[5] = bf16_hi(v.z);
    vals[6] = bf16_lo(v.w); vals[7] = bf16_hi(v.w);
  }
};

// f32: a 16-byte vector = 4 elements
template <>
struct Row<false> {
  static constexpr int kElems = 4;
  typedef f32x4 Raw;
  __device__ static Raw load_raw(const void* base, size_t row, int row_vecs, int c) {
    return __builtin_nontemporal_load(static_cast<const f32x4*>(base) + row * row_vecs + c);
  }
  __device__ static void unpack(const Raw& v, float* out) { out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w; }
  __device__ static void load(const void* base, size_t row, int row_vecs, int c, float* out) {
    unpack(load_raw(base, row, row_vecs, c), out);
  }
  __device__ static void store_round(void* base, size_t row, int row_vecs, int c, float* vals) {
    f32x4 v;
    v.x = vals[0]; v.y = vals[1]; v.z = vals[2]; v.w = vals[3];
    __builtin_nontemporal_store(v, static_cast<f32x4*>(base) + row * row_vecs + c);
  }
};

constexpr int kWave = 64;
constexpr int kPlanTokensPerBlock = 256;   // planner: one token per thread

}  // namespace occult
