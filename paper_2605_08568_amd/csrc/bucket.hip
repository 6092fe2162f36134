// a5: bucket prompts by identical rank subset, so that one launch (or one contiguous run of token tiles)
// serves one pattern (Sec. 4.3: rank patterns are shared across prompts).
//
// One workgroup, one lane per prompt (P <= 1024; the block is P rounded up to whole wavefronts).  Lane p
// reads its subset once and keeps a 64-bit signature of it in LDS; it then looks for the first earlier prompt
// with the same signature (LDS only) and confirms the match entry by entry, so equality is exact whatever the
// ids are.  Prompts that are their own first are pattern representatives, numbered by a prefix sum in arrival
// order; the stable permutation is a counting sort.  Integer work only, the result does not depend on
// scheduling.
#include "bucket.hpp"

namespace parse {

__global__ __launch_bounds__(1024) void bucket_patterns(const int32_t *__restrict__ subset, int P, int k, int stride,
                                                        int32_t *__restrict__ pattern_id, int32_t *__restrict__ perm,
                                                        int32_t *__restrict__ bucket_off,
                                                        int32_t *__restrict__ n_patterns, int32_t *__restrict__ rep) {
  bucket_body(subset, P, k, stride, pattern_id, perm, bucket_off, n_patterns, rep);
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
