// Constants and small device helpers shared by the bf16 prefill kernels (fused and two-launch forms).
#pragma once
#include "common.hpp"

namespace parse {

constexpr int PF_THREADS = 256;
constexpr int PF_BK = 64;            // reduction indices per staged X tile (4 matrix instructions deep)
constexpr int PF_XPAD = 8;           // bf16 of padding per LDS row: keeps 16-byte operand reads conflict-free
constexpr int PF_ZPAD = 8;
constexpr int PF_DEPTH = 8;          // reduction steps of factor operands in flight per wavefront

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
// two floats -> packed bfloat16 pair, round to nearest even (hardware conversion)
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}

// Workgroup ids are dealt round-robin over the 8 accelerator dies (XCDs), each with its own L2.  Token tiles
// are renumbered so that the tiles one die works on are consecutive: tiles of one prompt share a pattern, so
// they stream the same packed factors and hit in that die's L2 instead of each die fetching every pattern.
__device__ __forceinline__ int xcd_tile(int b, int nb) {
  const int per = nb / 8, rem = nb % 8, x = b % 8, i = b / 8;
  return x * per + min(x, rem) + i;
}

struct PfArgs {
  const uint16_t *X, *Vt_S, *Ut_S;
  uint16_t *Y;
  const int32_t *tok_offsets, *pattern_id;
  int n_patterns, rows, n, m, rS, P;
  // shared head (Sec. 4.4): the first sh_ranks of the rS selected ranks live once in Vt_sh / Ut_sh, the packed
  // per-pattern blocks hold the other rS - sh_ranks; 0 = everything per pattern
  const uint16_t *Vt_sh = nullptr, *Ut_sh = nullptr;
  int sh_ranks = 0;
};


}  // namespace parse
