// Body of the bucketing kernel (one workgroup, blockDim.x >= P a multiple of 64), shared by the stand-alone launch and
// the launch that also builds the prefill plan.
#pragma once
#include "common.hpp"

namespace parse {

constexpr int kBucketMaxK = 64;
constexpr int kBucketMaxP = 1024;

// inclusive scan of v[0..T) in LDS, T = blockDim.x a multiple of 64; every lane takes part
__device__ __forceinline__ void block_scan_inclusive(int32_t *v, int T) {
  const int p = threadIdx.x;
  for (int o = 1; o < T; o <<= 1) {
    const int add = (p >= o) ? v[p - o] : 0;
    __syncthreads();
    v[p] += add;
    __syncthreads();
  }
}

__device__ __forceinline__ void bucket_body(const int32_t *__restrict__ subset, int P, int k, int stride,
                                                        int32_t *__restrict__ pattern_id, int32_t *__restrict__ perm,
                                                        int32_t *__restrict__ bucket_off,
                                                        int32_t *__restrict__ n_patterns, int32_t *__restrict__ rep) {
  __shared__ unsigned long long sig[1024];
  __shared__ int32_t scan[1024];   // inclusive scan of "is representative", later of the pattern sizes
  __shared__ int32_t pid[1024];
  __shared__ int32_t cnt[1025];
  const int p = threadIdx.x, T = blockDim.x;
  const int32_t *mine = subset + (size_t)min(p, P - 1) * stride;
  unsigned long long h = 0x9E3779B97F4A7C15ull;
  for (int i = 0; i < k; ++i) {   // independent loads, then a sequential mix
    h ^= (unsigned long long)(uint32_t)mine[i];
    h *= 0xFF51AFD7ED558CCDull;
    h ^= h >> 29;
  }
  sig[p] = h;
  cnt[p] = 0;
  if (p == 0) cnt[T] = 0;
  __syncthreads();
  int first = p;
  if (p < P) {
    for (int q = 0; q < p; ++q) {
      if (sig[q] != h) continue;
      bool same = true;
      for (int i = 0; i < k; ++i) same = same && (subset[(size_t)q * stride + i] == mine[i]);
      if (same) { first = q; break; }
    }
  }
  const int is_rep = (p < P && first == p) ? 1 : 0;
  scan[p] = is_rep;
  __syncthreads();
  block_scan_inclusive(scan, T);
  const int npat = scan[T - 1];
  if (p < P) pid[p] = scan[first] - 1;   // representative's exclusive rank
  __syncthreads();
  if (p < P) atomicAdd(&cnt[pid[p] + 1], 1);
  __syncthreads();
  scan[p] = cnt[p + 1];                  // size of pattern p
  __syncthreads();
  block_scan_inclusive(scan, T);
  // scan[j] = number of prompts in patterns 0..j  =>  bucket_off[j+1]
  if (p < P) {
    const int j = pid[p];
    const int base = j > 0 ? scan[j - 1] : 0;
    int rank = 0;
    for (int q = 0; q < p; ++q) rank += (pid[q] == j) ? 1 : 0;
    perm[base + rank] = p;
    pattern_id[p] = j;
    if (is_rep) rep[j] = p;
    bucket_off[p + 1] = (p < npat) ? scan[p] : P;
    if (p >= npat) rep[p] = -1;
  }
  if (p == 0) {
    bucket_off[0] = 0;
    *n_patterns = npat;
  }
}

}  // namespace parse
