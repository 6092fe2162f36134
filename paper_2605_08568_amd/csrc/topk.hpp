// Router scoring and top-k selection shared by the route and cache kernels.
#pragma once
#include "common.hpp"

namespace parse {

// Scores s_g = <Wr[g], e> for g in [0, G): e lives in LDS (d floats, d % 4 == 0), each of the block's
// wavefronts takes every nwaves-th group and reduces across its 64 lanes.  Result in s_lds[G]; ends
// with a barrier.
__device__ __forceinline__ void block_router_scores(const float *__restrict__ Wr, const float *e_lds,
                                                    int d, int G, float *s_lds) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  for (int g = wave; g < G; g += nwaves) {
    const float4 *w4 = reinterpret_cast<const float4 *>(Wr + (size_t)g * d);
    const float4 *e4 = reinterpret_cast<const float4 *>(e_lds);
    float acc = 0.f;
#pragma unroll 8
    for (int c = lane; c < d / 4; c += 64) {
      const float4 w = w4[c];
      const float4 e = e4[c];
      acc += w.x * e.x + w.y * e.y + w.z * e.z + w.w * e.w;
    }
    acc = wave_sum(acc);
    if (lane == 0) s_lds[g] = acc;
  }
  __syncthreads();
}

// Top-k of s_lds[0..G), G <= 64, by ONE wavefront (call with the 64 lanes of wave 0): groups 0..n_shared-1 are
// always taken (the shared head, Sec. 4.4); lane g >= n_shared ranks its score among the other routed groups
// (larger first, equal scores by lower id) and is taken when its rank is below k - n_shared; the k ids are
// written ascending to out[0..k).
__device__ __forceinline__ void wave_topk_ascending(const float *s_lds, int G, int k, int32_t *out, int n_shared = 0) {
  const int g = threadIdx.x & 63;
  bool sel = false;
  if (g < G) {
    if (g < n_shared) {
      sel = g < k;
    } else {
      const float s = s_lds[g];
      int rank = 0;
      for (int h = n_shared; h < G; ++h) {
        const float t = s_lds[h];
        rank += (t > s || (t == s && h < g)) ? 1 : 0;
      }
      sel = rank < k - n_shared;
    }
  }
  const unsigned long long mask = __ballot(sel);
  if (sel) {
    const int pos = __popcll(mask & ((1ull << g) - 1ull));
    if (pos < k) out[pos] = g;
  }
}

}  // namespace parse
