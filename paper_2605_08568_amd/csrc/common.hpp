// Shared host/device helpers of the gfx950 kernels (internal; the public surface is include/parse.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "parse.h"

namespace parse {

constexpr int kWave = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// bfloat16 bit pattern <-> float.  Rounding: nearest even (the format's standard conversion).
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Sum / max across the 64 lanes of a wavefront (butterfly; every lane gets the result).
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Last HIP error text of this thread, for parse_last_hip_error().
void set_hip_error(hipError_t e, const char *where);

#define PARSE_HIP_TRY(expr)                         \
  do {                                              \
    hipError_t _e = (expr);                         \
    if (_e != hipSuccess) {                         \
      ::parse::set_hip_error(_e, #expr);            \
      return PARSE_EHIP;                            \
    }                                               \
  } while (0)

// A launch with more than 64 KiB of dynamic LDS needs the kernel's limit raised first (gfx950 has 160 KiB per CU).
// Only the rare large shapes take this path, so the attribute is simply set again on each such call.
#define PARSE_ALLOW_LDS(kernel, bytes)                                                                            \
  do {                                                                                                            \
    if ((size_t)(bytes) > (size_t)65536)                                                                          \
      PARSE_HIP_TRY(hipFuncSetAttribute((const void *)(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(bytes))); \
  } while (0)

#define PARSE_LAUNCH_CHECK()                        \
  do {                                              \
    hipError_t _e = hipGetLastError();              \
    if (_e != hipSuccess) {                         \
      ::parse::set_hip_error(_e, "kernel launch");  \
      return PARSE_EHIP;                            \
    }                                               \
  } while (0)

static inline bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }
static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int elem_size(int dtype) { return dtype == PARSE_BF16 ? 2 : 4; }

// Host-side check of a parse_layer: returns PARSE_OK or the status to hand back.
int check_layer(const parse_layer *L);

}  // namespace parse

namespace parse {
// The same answer as prompt_of_row below, found by a whole wavefront at once (every lane must call it with the same
// row): for P <= 64 lane l reads tok_offsets[l] and the lanes vote, one memory round trip instead of log2(P)
// dependent ones; longer tables fall back to the binary search.
__device__ __forceinline__ int prompt_of_row(const int32_t *__restrict__ tok_offsets, int P, int row);
__device__ __forceinline__ int prompt_of_row_wave(const int32_t *__restrict__ tok_offsets, int P, int row) {
  if (P > 64) return prompt_of_row(tok_offsets, P, row);
  const int lane = threadIdx.x & 63;
  const bool le = lane < P && tok_offsets[lane] <= row;
  const int n = __popcll(__ballot(le));
  return n > 0 ? n - 1 : 0;
}

// Largest p in [0, P) with tok_offsets[p] <= row (tok_offsets ascending, tok_offsets[0] == 0).
__device__ __forceinline__ int prompt_of_row(const int32_t *__restrict__ tok_offsets, int P, int row) {
  int lo = 0, hi = P - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (tok_offsets[mid] <= row) lo = mid; else hi = mid - 1;
  }
  return lo;
}
}  // namespace parse
