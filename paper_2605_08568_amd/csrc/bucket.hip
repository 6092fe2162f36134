// a5: bucket prompts by identical rank subset, so that one launch (or one contiguous run of token tiles)
// serves one pattern (Sec. 4.3: rank patterns are shared across prompts).
//
// One workgroup, one lane per prompt (P <= 1024; the block is P rounded up to whole wavefronts).  Lane p
// reads its subset once and keeps a 64-bit signature of it in LDS; it then looks for the first earlier prompt
// with the same signature (LDS only) and confirms the match entry by entry, so equality is exact whatever the
// ids are.  Prompts that are their own first are pattern representatives, numbered by a prefix sum in arrival
// order; the stable permutation is a counting sort.  Integer work only, the result does not depend on
// scheduling.
#include "common.hpp"

namespace parse {

constexpr int kBucketMaxK = 64;

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

__global__ __launch_bounds__(1024) void bucket_patterns(const int32_t *__restrict__ subset, int P, int k, int stride,
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

using namespace parse;

extern "C" int parse_bucket_patterns(const int32_t *subset, int32_t P, int32_t k, int32_t subset_stride,
                                     int32_t *pattern_id, int32_t *perm, int32_t *bucket_off, int32_t *n_patterns,
                                     int32_t *rep, parse_stream stream) {
  if (!subset || !pattern_id || !perm || !bucket_off || !n_patterns || !rep) return PARSE_EINVAL;
  if (P <= 0 || k <= 0) return PARSE_EINVAL;
  if (P > 1024 || k > 64 || subset_stride < k) return PARSE_ESHAPE;
  hipLaunchKernelGGL(bucket_patterns, dim3(1), dim3((P + 63) / 64 * 64), 0, (hipStream_t)stream, subset, P, k, subset_stride,
                     pattern_id, perm, bucket_off, n_patterns, rep);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}
