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

constexpr int kWave = 64;
constexpr int kPlanTokensPerBlock = 256;   // planner: one token per thread

}  // namespace occult
