// a1 + a2: prompt pooling and the linear router with top-k (Sec. 4.1, Eq. 5).
//
// Two launches, both deterministic:
//   pool_partial  grid (column blocks of 64 lanes x 16 bytes, Q row slices, P prompts): the rows of a prompt are
//                 dealt round robin to the wavefronts of its Q workgroups, 16 rows in flight per wavefront; the
//                 four wavefronts of a workgroup add up through LDS in wavefront order; fp32 partial sums per
//                 slice, rows streamed once.
//   route_finish  one block per prompt: adds the Q partials in slice order, divides by the length,
//                 scores the G groups (one wavefront per group, butterfly reduction) and selects the
//                 top k with a rank count inside one wavefront.
#include "common.hpp"
#include "topk.hpp"

namespace parse {

constexpr int kPoolThreads = 256, kPoolWaves = kPoolThreads / 64;

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

template <bool BF16>
__global__ __launch_bounds__(kPoolThreads) void pool_partial(const void *__restrict__ X, int rows, int d,
                                                             const int32_t *__restrict__ tok_offsets,
                                                             int Q, float *__restrict__ partial) {
  constexpr int PER = BF16 ? 8 : 4;  // columns per lane = 16 bytes
  constexpr int U = 16;              // rows a wavefront has in flight
  __shared__ float red[kPoolWaves - 1][PER][64];
  const int p = blockIdx.z, q = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int c0 = (blockIdx.x * 64 + lane) * PER;
  const bool in = c0 < d;
  const int a = clampi(tok_offsets[p], 0, rows);
  const int b = clampi(tok_offsets[p + 1], a, rows);
  // the rows of a prompt are dealt round robin to the Q * kPoolWaves wavefronts that share a column block: at any
  // moment they read a window of consecutive rows
  const int r0 = a + q * kPoolWaves + wave, r1 = b, rstep = Q * kPoolWaves;
  float acc[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) acc[i] = 0.f;
  // U rows at a time: all of them are requested before the first is added (left to itself the compiler waits for every
  // row before it asks for the next); rows past the end re-read the wavefront's last row and are not added; the adds
  // run in row order.  Lanes past the last column re-read the last piece of the row; their sums are not stored.
  const char *xb = reinterpret_cast<const char *>(X) + (size_t)min(c0, d - PER) * (BF16 ? 2 : 4);
  const size_t row_bytes = (size_t)d * (BF16 ? 2 : 4);
  for (int r = r0; r < r1; r += rstep * U) {
    const int rlast = r + ((r1 - 1 - r) / rstep) * rstep;
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = *reinterpret_cast<const u32x4 *>(xb + (size_t)min(r + u * rstep, rlast) * row_bytes);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (r + u * rstep < r1) {       // uniform
        if constexpr (BF16) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[2 * i] += __uint_as_float(v[u][i] << 16);
            acc[2 * i + 1] += __uint_as_float(v[u][i] & 0xFFFF0000u);
          }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[i] += __uint_as_float(v[u][i]);
        }
      }
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < PER; ++i) red[wave - 1][i][lane] = acc[i];
  }
  __syncthreads();
  if (wave == 0 && in) {
    for (int w = 0; w < kPoolWaves - 1; ++w)
#pragma unroll
      for (int i = 0; i < PER; ++i) acc[i] += red[w][i][lane];
    float *dst = partial + ((size_t)p * Q + q) * d + c0;
#pragma unroll
    for (int i = 0; i < PER; i += 4) *reinterpret_cast<float4 *>(dst + i) = float4{acc[i], acc[i + 1], acc[i + 2], acc[i + 3]};
  }
}

constexpr int kFinishThreads = 1024;

__global__ __launch_bounds__(kFinishThreads) void route_finish(const float *__restrict__ partial, int Q, int rows, int d,
                                                               const int32_t *__restrict__ tok_offsets,
                                                               const float *__restrict__ Wr, int G, int k,
                                                               int32_t *__restrict__ subset_out, int subset_stride,
                                                               float *__restrict__ scores_out,
                                                               float *__restrict__ emb_out, int n_shared) {
  extern __shared__ float lds[];
  float *e = lds;          // [d]
  float *s = lds + d;      // [64]
  const int p = blockIdx.x;
  const int a = clampi(tok_offsets[p], 0, rows);
  const int b = clampi(tok_offsets[p + 1], a, rows);
  const float inv = (b > a) ? 1.0f / (float)(b - a) : 0.f;
  // four columns per lane, the Q slice partials added in slice order (independent loads, fixed order of adds)
  for (int c = threadIdx.x * 4; c < d; c += kFinishThreads * 4) {
    const float *src = partial + (size_t)p * Q * d + c;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int q = 0; q < Q; ++q) {
      const float4 v = *reinterpret_cast<const float4 *>(src + (size_t)q * d);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    *reinterpret_cast<float4 *>(e + c) = acc;
    if (emb_out) *reinterpret_cast<float4 *>(emb_out + (size_t)p * d + c) = acc;
  }
  __syncthreads();
  block_router_scores(Wr, e, d, G, s);
  if (scores_out)
    for (int g = threadIdx.x; g < G; g += blockDim.x) scores_out[(size_t)p * G + g] = s[g];
  if (threadIdx.x < 64) wave_topk_ascending(s, G, k, subset_out + (size_t)p * subset_stride, n_shared);
}

// Slices per prompt: about two workgroups per compute unit, a slice of at least 32 rows (8 per wavefront), at most
// 32 slices.
static int pool_slices(int rows, int P, int d, bool bf16) {
  const int per_block = 64 * (bf16 ? 8 : 4);
  const int colblocks = (d + per_block - 1) / per_block;
  long long want = (512 + (long long)P * colblocks - 1) / ((long long)P * colblocks);
  long long avg = rows / (P > 0 ? P : 1);
  long long by_len = avg / 32 > 0 ? avg / 32 : 1;
  long long q = want < by_len ? want : by_len;
  if (q > 32) q = 32;
  if (q < 1) q = 1;
  return (int)q;
}

// Launches pool_partial into `partial` ([P][Q][d] floats, Q returned); shared with the rank-granular router.
int launch_pool_partials(const void *X, int xdtype, int rows, const int32_t *tok_offsets, int P, int d, float *partial,
                         int *Q_out, hipStream_t s) {
  const bool bf16 = xdtype == PARSE_BF16;
  const int Q = pool_slices(rows, P, d, bf16);
  const int per_block = 64 * (bf16 ? 8 : 4);
  dim3 grid((d + per_block - 1) / per_block, Q, P);
  if (bf16)
    hipLaunchKernelGGL(pool_partial<true>, grid, dim3(kPoolThreads), 0, s, X, rows, d, tok_offsets, Q, partial);
  else
    hipLaunchKernelGGL(pool_partial<false>, grid, dim3(kPoolThreads), 0, s, X, rows, d, tok_offsets, Q, partial);
  PARSE_LAUNCH_CHECK();
  *Q_out = Q;
  return PARSE_OK;
}

int launch_pool_finish(const float *partial, int Q, int rows, int d, const int32_t *tok_offsets, int P, float *emb,
                       hipStream_t s);   // with the rank-granular router

}  // namespace parse

using namespace parse;

extern "C" {

size_t parse_route_workspace_bytes(int32_t rows, int32_t P, int32_t d) {
  if (rows <= 0 || P <= 0 || d <= 0) return 0;
  // the slice count does not depend on the dtype beyond the column-block count; size for the larger one
  const int q = pool_slices(rows, P, d, false) > pool_slices(rows, P, d, true) ? pool_slices(rows, P, d, false)
                                                                                  : pool_slices(rows, P, d, true);
  return round_up((size_t)P * q * d * sizeof(float), 256);
}

int parse_pool(const void *X, int32_t xdtype, int32_t rows, const int32_t *tok_offsets, int32_t P, int32_t d,
               float *emb_out, void *workspace, size_t workspace_bytes, parse_stream stream) {
  if (!X || !tok_offsets || !emb_out) return PARSE_EINVAL;
  if (xdtype != PARSE_F32 && xdtype != PARSE_BF16) return PARSE_EINVAL;
  if (rows <= 0 || P <= 0 || d <= 0) return PARSE_EINVAL;
  if (d > 16384 || P > rows) return PARSE_ESHAPE;
  if (d % 8 != 0) return PARSE_EALIGN;
  if (!aligned16(X) || !aligned16(emb_out) || !aligned16(workspace)) return PARSE_EALIGN;
  if (!workspace || workspace_bytes < parse_route_workspace_bytes(rows, P, d)) return PARSE_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  float *partial = reinterpret_cast<float *>(workspace);
  int Q = 0;
  const int st = launch_pool_partials(X, xdtype, rows, tok_offsets, P, d, partial, &Q, s);
  if (st != PARSE_OK) return st;
  return launch_pool_finish(partial, Q, rows, d, tok_offsets, P, emb_out, s);
}

int parse_route(const void *X, int32_t xdtype, int32_t rows, const int32_t *tok_offsets, int32_t P, int32_t d,
                const float *Wr, int32_t G, int32_t k, int32_t *subset_out, int32_t subset_stride,
                float *scores_out, float *emb_out, void *workspace, size_t workspace_bytes,
                parse_stream stream) {
  return parse_route_shared(X, xdtype, rows, tok_offsets, P, d, Wr, G, k, 0, subset_out, subset_stride, scores_out,
                            emb_out, workspace, workspace_bytes, stream);
}

int parse_route_shared(const void *X, int32_t xdtype, int32_t rows, const int32_t *tok_offsets, int32_t P, int32_t d,
                       const float *Wr, int32_t G, int32_t k, int32_t n_shared, int32_t *subset_out,
                       int32_t subset_stride, float *scores_out, float *emb_out, void *workspace,
                       size_t workspace_bytes, parse_stream stream) {
  if (!X || !tok_offsets || !Wr || !subset_out) return PARSE_EINVAL;
  if (xdtype != PARSE_F32 && xdtype != PARSE_BF16) return PARSE_EINVAL;
  if (rows <= 0 || P <= 0 || d <= 0 || G <= 0 || k <= 0) return PARSE_EINVAL;
  if (n_shared < 0) return PARSE_EINVAL;
  if (k > G || G > 64 || d > 16384 || P > rows || subset_stride < k || n_shared > k) return PARSE_ESHAPE;
  if (d % 8 != 0) return PARSE_EALIGN;
  if (!aligned16(X) || !aligned16(Wr) || !aligned16(workspace)) return PARSE_EALIGN;
  if (emb_out && !aligned16(emb_out)) return PARSE_EALIGN;
  if (!workspace || workspace_bytes < parse_route_workspace_bytes(rows, P, d)) return PARSE_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  float *partial = reinterpret_cast<float *>(workspace);
  int Q = 0;
  const int st = launch_pool_partials(X, xdtype, rows, tok_offsets, P, d, partial, &Q, s);
  if (st != PARSE_OK) return st;
  const size_t lds = (size_t)(d + 64) * sizeof(float);
  PARSE_ALLOW_LDS(route_finish, lds);
  hipLaunchKernelGGL(route_finish, dim3(P), dim3(kFinishThreads), lds, s, partial, Q, rows, d, tok_offsets, Wr, G, k,
                     subset_out, subset_stride, scores_out, emb_out, n_shared);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // extern "C"
