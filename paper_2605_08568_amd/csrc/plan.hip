// Execution plan of one prefill batch (Sec. 4.3: prompts that share a rank pattern are executed together; Sec. 4.4:
// one contiguous factor block per pattern).  The token rows of all prompts are renumbered so that the rows of
// one pattern are consecutive ("virtual rows", prompts of a pattern in arrival order) and every pattern starts on a
// 256-row boundary.  A 256-row tile of virtual rows therefore belongs to exactly one pattern, whatever the prompt
// lengths are: the tile kernels never split a tile between patterns and never redo a tile per prompt segment; the
// only waste is the padding at the end of each pattern (< 256 rows per pattern present in the batch).
// The plan depends only on (tok_offsets, pattern_id): one plan serves every layer of a model for that batch.
//
// Layout of the plan (int32 words, device memory, caller-owned):
//   [0] number of 256-row virtual tiles  [1] virtual rows (= 256 * [0])  [2] 256  [3] capacity in tiles  [4..15] 0
//   [16 .. 16+cap)            pattern of each virtual tile (-1: prompts whose pattern id is out of range -> zero rows)
//   [16+cap16 .. +256*cap)    rowmap: actual token row of each virtual row, -1 for padding     (cap16 = cap rounded up to 16)
#include "bucket.hpp"
#include "common.hpp"

namespace parse {

constexpr int PLAN_VT = 256;          // rows per virtual tile
constexpr int PLAN_HDR = 16;
constexpr int PLAN_MAX_P = 2048;
constexpr int PLAN_MAX_PATTERNS = 2048;
constexpr int PLAN_THREADS = 256;

static inline int plan_capacity_tiles(int rows, int P, int n_patterns) {
  const int buckets = (P < n_patterns + 1) ? P : n_patterns + 1;   // patterns present, plus one bucket of invalid ids
  return (rows + PLAN_VT - 1) / PLAN_VT + buckets;
}
static inline size_t plan_words(int cap) { return (size_t)PLAN_HDR + (size_t)((cap + 15) / 16 * 16) + (size_t)cap * PLAN_VT; }

// Every workgroup works out the (small) per-pattern and per-prompt tables in its own LDS -- integer work, the same in
// every workgroup -- and then fills its share of the row map.
// (block, nblocks) = this workgroup's place among the workgroups that build the plan.
__device__ __forceinline__ void plan_body(const int32_t *__restrict__ tok_offsets, const int32_t *__restrict__ pattern_id,
                                          int P, int rows, int NP, int cap, int32_t *__restrict__ plan, int block,
                                          int nblocks) {
  __shared__ int32_t cnt[PLAN_MAX_PATTERNS + 1];     // rows of each pattern (index NP: invalid ids); later: running fill
  __shared__ int32_t base[PLAN_MAX_PATTERNS + 2];    // first virtual row of each pattern
  __shared__ int32_t vstart[PLAN_MAX_P];             // first virtual row of each prompt
  __shared__ int32_t offs[PLAN_MAX_P + 1];           // tok_offsets clamped to [0, rows] and made non-decreasing per prompt
  __shared__ int32_t pids[PLAN_MAX_P];               // pattern of each prompt, NP for ids out of range
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  int32_t *tile_pat = plan + PLAN_HDR;
  int32_t *rowmap = plan + PLAN_HDR + (cap + 15) / 16 * 16;
  const int max_v = cap * PLAN_VT;
  // one pass over the two input arrays; everything after it works on LDS
  for (int p = tid; p <= P; p += PLAN_THREADS) {
    const int a = tok_offsets[p];
    offs[p] = a < 0 ? 0 : (a > rows ? rows : a);
    if (p < P) {
      const int v = pattern_id[p];
      pids[p] = (v >= 0 && v < NP) ? v : NP;
    }
  }
  auto prompt_len = [&](int p) -> int { return max(offs[p + 1] - offs[p], 0); };
  auto prompt_pid = [&](int p) -> int { return pids[p]; };
  for (int i = tid; i <= NP; i += PLAN_THREADS) cnt[i] = 0;
  __syncthreads();   // also: offs / pids are complete
  for (int p = tid; p < P; p += PLAN_THREADS) atomicAdd(&cnt[prompt_pid(p)], prompt_len(p));   // integer sums: order-free
  __syncthreads();
  // exclusive prefix of the padded pattern sizes: one wavefront, 64 patterns per step
  if (tid < 64) {
    int carry = 0;
    for (int i0 = 0; i0 <= NP; i0 += 64) {
      const int i = i0 + lane;
      const int padded = (i <= NP) ? (cnt[i] + PLAN_VT - 1) / PLAN_VT * PLAN_VT : 0;
      int incl = padded;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
      }
      if (i <= NP) base[i] = carry + incl - padded;
      carry += __shfl(incl, 63, 64);
    }
    if (lane == 0) base[NP + 1] = carry;
  }
  __syncthreads();
  for (int i = tid; i <= NP; i += PLAN_THREADS) cnt[i] = 0;    // now: rows of the pattern placed so far
  __syncthreads();
  // prompts in arrival order, 64 at a time: a prompt starts after the earlier prompts of its pattern
  if (tid < 64) {
    for (int p0 = 0; p0 < P; p0 += 64) {
      const int p = p0 + lane;
      const int pid = p < P ? prompt_pid(p) : -1;
      const int len = p < P ? prompt_len(p) : 0;
      int before = 0;
      const int n_here = min(64, P - p0);          // prompts in this chunk (uniform)
      for (int l2 = 0; l2 + 1 < n_here; ++l2) {
        const int opid = __shfl(pid, l2, 64), olen = __shfl(len, l2, 64);
        if (l2 < lane && opid == pid) before += olen;
      }
      if (p < P) vstart[p] = base[pid] + cnt[pid] + before;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      if (p < P) atomicAdd(&cnt[pid], len);
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    }
  }
  __syncthreads();
  const int total = min(base[NP + 1], max_v);
  const int gid = block * PLAN_THREADS + tid, gstride = nblocks * PLAN_THREADS;
  if (gid == 0) {
    plan[0] = total / PLAN_VT; plan[1] = total; plan[2] = PLAN_VT; plan[3] = cap;
    for (int i = 4; i < PLAN_HDR; ++i) plan[i] = 0;
  }
  // pattern of each tile, and the padding rows at the end of each pattern
  for (int i = block; i <= NP; i += nblocks) {
    const int b0 = base[i], b1 = base[i + 1];
    if (b1 == b0) continue;
    for (int t = b0 / PLAN_VT + tid; t < b1 / PLAN_VT; t += PLAN_THREADS)
      if (t < cap) tile_pat[t] = (i < NP) ? i : -1;
    for (int v = b0 + cnt[i] + tid; v < b1; v += PLAN_THREADS)
      if (v < max_v) rowmap[v] = -1;
  }
  // every real row: its prompt (binary search in LDS), then its place in the pattern's run
  for (int r = gid; r < rows; r += gstride) {
    int lo = 0, hi = P - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (offs[mid] <= r) lo = mid; else hi = mid - 1;
    }
    const int within = r - offs[lo];
    if (within >= 0 && within < prompt_len(lo)) {
      const int v = vstart[lo] + within;
      if (v >= 0 && v < max_v) rowmap[v] = r;
    }
  }
}

__global__ __launch_bounds__(PLAN_THREADS) void plan_build(const int32_t *__restrict__ tok_offsets,
                                                           const int32_t *__restrict__ pattern_id, int P, int rows,
                                                           int NP, int cap, int32_t *__restrict__ plan) {
  plan_body(tok_offsets, pattern_id, P, rows, NP, cap, plan, blockIdx.x, gridDim.x);
}

// The plan and the buckets of a batch in one launch (they depend on the same probe results and not on each other): the
// last workgroup buckets the prompts, the others build the plan.  P <= PLAN_THREADS (one lane per prompt in the bucketing).
struct BucketArgs {
  const int32_t *subset;
  int k, stride;
  int32_t *pattern_id, *perm, *bucket_off, *n_patterns, *rep;
};
__global__ __launch_bounds__(PLAN_THREADS) void bucket_and_plan(BucketArgs b, const int32_t *__restrict__ tok_offsets,
                                                                const int32_t *__restrict__ pattern_id, int P, int rows,
                                                                int NP, int cap, int32_t *__restrict__ plan) {
  if (blockIdx.x + 1 == gridDim.x)     // uniform
    bucket_body(b.subset, P, b.k, b.stride, b.pattern_id, b.perm, b.bucket_off, b.n_patterns, b.rep);
  else
    plan_body(tok_offsets, pattern_id, P, rows, NP, cap, plan, blockIdx.x, gridDim.x - 1);
}

size_t prefill_plan_bytes(int rows, int P, int n_patterns) {
  return round_up(plan_words(plan_capacity_tiles(rows, P, n_patterns)) * sizeof(int32_t), 256);
}
int prefill_plan_capacity(int rows, int P, int n_patterns) { return plan_capacity_tiles(rows, P, n_patterns); }
bool prefill_plan_supported(int P, int n_patterns) { return P <= PLAN_MAX_P && n_patterns <= PLAN_MAX_PATTERNS; }

static int plan_grid(int rows) {
  const int grid = (rows + 4 * PLAN_THREADS - 1) / (4 * PLAN_THREADS);   // about four rows per thread
  return grid < 1 ? 1 : (grid > 128 ? 128 : grid);
}

int build_prefill_plan(const int32_t *tok_offsets, const int32_t *pattern_id, int P, int rows, int n_patterns,
                       int32_t *plan, hipStream_t s) {
  const int cap = plan_capacity_tiles(rows, P, n_patterns);
  const int grid = plan_grid(rows);
  hipLaunchKernelGGL(plan_build, dim3(grid), dim3(PLAN_THREADS), 0, s, tok_offsets, pattern_id, P, rows, n_patterns, cap, plan);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // namespace parse

using namespace parse;

extern "C" {

size_t parse_prefill_plan_bytes(int32_t rows, int32_t P, int32_t n_patterns) {
  if (rows <= 0 || P <= 0 || n_patterns <= 0) return 0;
  return prefill_plan_bytes(rows, P, n_patterns);
}

int parse_prefill_plan(const int32_t *tok_offsets, const int32_t *pattern_id, int32_t P, int32_t rows,
                       int32_t n_patterns, void *plan, size_t plan_bytes, parse_stream stream) {
  if (!tok_offsets || !pattern_id || !plan) return PARSE_EINVAL;
  if (P <= 0 || rows <= 0 || n_patterns <= 0) return PARSE_EINVAL;
  if (P > rows || !prefill_plan_supported(P, n_patterns)) return PARSE_ESHAPE;
  if (!aligned16(plan)) return PARSE_EALIGN;
  if (plan_bytes < prefill_plan_bytes(rows, P, n_patterns)) return PARSE_EWORKSPACE;
  return build_prefill_plan(tok_offsets, pattern_id, P, rows, n_patterns, (int32_t *)plan, (hipStream_t)stream);
}

int parse_bucket_and_plan(const int32_t *subset, int32_t P, int32_t k, int32_t subset_stride, int32_t *pattern_id_out,
                          int32_t *perm, int32_t *bucket_off, int32_t *n_patterns_out, int32_t *rep,
                          const int32_t *tok_offsets, const int32_t *plan_pattern_id, int32_t rows, int32_t n_patterns,
                          void *plan, size_t plan_bytes, parse_stream stream) {
  if (!subset || !pattern_id_out || !perm || !bucket_off || !n_patterns_out || !rep) return PARSE_EINVAL;
  if (!tok_offsets || !plan_pattern_id || !plan) return PARSE_EINVAL;
  if (P <= 0 || k <= 0 || rows <= 0 || n_patterns <= 0) return PARSE_EINVAL;
  if (P > kBucketMaxP || k > kBucketMaxK || subset_stride < k) return PARSE_ESHAPE;
  if (P > rows || !prefill_plan_supported(P, n_patterns)) return PARSE_ESHAPE;
  if (!aligned16(plan)) return PARSE_EALIGN;
  if (plan_bytes < prefill_plan_bytes(rows, P, n_patterns)) return PARSE_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  if (P > PLAN_THREADS) {     // more prompts than lanes of a plan workgroup: the two launches of the separate calls
    const int st = parse_bucket_patterns(subset, P, k, subset_stride, pattern_id_out, perm, bucket_off, n_patterns_out, rep, stream);
    if (st != PARSE_OK) return st;
    return build_prefill_plan(tok_offsets, plan_pattern_id, P, rows, n_patterns, (int32_t *)plan, s);
  }
  const BucketArgs b{subset, k, subset_stride, pattern_id_out, perm, bucket_off, n_patterns_out, rep};
  hipLaunchKernelGGL(bucket_and_plan, dim3(plan_grid(rows) + 1), dim3(PLAN_THREADS), 0, s, b, tok_offsets, plan_pattern_id, P,
                     rows, n_patterns, plan_capacity_tiles(rows, P, n_patterns), (int32_t *)plan);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // extern "C"
