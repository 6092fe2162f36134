// Rank-granular routing: the paper's own formulation (Sec. 4.1, Eq. 4-5) -- every rank-1 component is an expert,
// the router maps the prompt embedding to one score per rank (R^d -> R^{r_max}) and the K best ranks are active.
// The grouped path elsewhere in this library is the special case of contiguous groups; here
//   route_ranks  pool (shared with the grouped router) -> embedding -> scores = Wr e for thousands of ranks, a
//                bandwidth-bound skinny product that reads Wr once per block of 8 prompts -> exact top-K by radix
//                select over the score bits (ties to the lower rank id), ids written ascending;
//   pack_ranks   the K selected rank rows of a row-major bf16 layer are gathered and written straight into
//                matrix-core operand order (the memory aggregation of Sec. 4.4 for scattered single ranks: K
//                row reads of n*2 / m*2 bytes become one contiguous block per pattern), after which the
//                prefill kernels run unchanged with r_S = K.
#include "common.hpp"

namespace parse {

int launch_pool_partials(const void *X, int xdtype, int rows, const int32_t *tok_offsets, int P, int d, float *partial,
                         int *Q_out, hipStream_t s);

constexpr int RK_MAXG = 8192;        // ranks the selection kernel holds in LDS
constexpr int RK_PB = 8;             // prompts per scoring workgroup
constexpr int RK_RPW = 2;            // router rows per wavefront
constexpr int RK_ROWS = 4 * RK_RPW;  // router rows per scoring workgroup

// e[p][:] = (sum of the Q slice partials, in slice order) / prompt length.  grid (ceil(d/1024), P), block 256.
__global__ __launch_bounds__(256) void pool_finish(const float *__restrict__ partial, int Q, int rows, int d,
                                                   const int32_t *__restrict__ tok_offsets, float *__restrict__ emb) {
  const int p = blockIdx.y;
  const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c >= d) return;
  int a = tok_offsets[p], b = tok_offsets[p + 1];
  a = a < 0 ? 0 : (a > rows ? rows : a);
  b = b < a ? a : (b > rows ? rows : b);
  const float inv = (b > a) ? 1.0f / (float)(b - a) : 0.f;
  const float *src = partial + (size_t)p * Q * d + c;
  float4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
  for (int q = 0; q < Q; ++q) {
    const float4 v = *reinterpret_cast<const float4 *>(src + (size_t)q * d);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
  *reinterpret_cast<float4 *>(emb + (size_t)p * d + c) = acc;
}

// Shared with the embedding-only entry point.
int launch_pool_finish(const float *partial, int Q, int rows, int d, const int32_t *tok_offsets, int P, float *emb,
                       hipStream_t s) {
  hipLaunchKernelGGL(pool_finish, dim3((d + 1023) / 1024, P), dim3(256), 0, s, partial, Q, rows, d, tok_offsets, emb);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

// scores[p][g] = <Wr[g], e_p>.  grid (ceil(G/8), ceil(P/8)), block 256: wavefront w owns rows 2w, 2w+1 of the
// block for the 8 prompts of the block.  Pure streaming, no LDS and no barrier: a lane reads 16 bytes of each of
// its two router rows and of the 8 embeddings (cache-resident, 16 KB each) per 256-column step, four steps in
// flight; every lane keeps 2 x 8 partial sums and the 64 lanes are added at the end (fixed order: same inputs,
// same bits).
__global__ __launch_bounds__(256) void rank_scores(const float *__restrict__ Wr, const float *__restrict__ emb, int G,
                                                   int d, int P, float *__restrict__ scores) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g0 = blockIdx.x * RK_ROWS + wave * RK_RPW, p0 = blockIdx.y * RK_PB;
  float acc[RK_RPW][RK_PB];
#pragma unroll
  for (int r = 0; r < RK_RPW; ++r)
#pragma unroll
    for (int p = 0; p < RK_PB; ++p) acc[r][p] = 0.f;
  const float *wrow[RK_RPW], *erow[RK_PB];
#pragma unroll
  for (int r = 0; r < RK_RPW; ++r) wrow[r] = Wr + (size_t)min(g0 + r, G - 1) * d;
#pragma unroll
  for (int p = 0; p < RK_PB; ++p) erow[p] = emb + (size_t)min(p0 + p, P - 1) * d;
#pragma unroll 4
  for (int c = lane * 4; c < d; c += 256) {
    float4 w[RK_RPW], e[RK_PB];
#pragma unroll
    for (int r = 0; r < RK_RPW; ++r) w[r] = *reinterpret_cast<const float4 *>(wrow[r] + c);
#pragma unroll
    for (int p = 0; p < RK_PB; ++p) e[p] = *reinterpret_cast<const float4 *>(erow[p] + c);
#pragma unroll
    for (int p = 0; p < RK_PB; ++p)
#pragma unroll
      for (int r = 0; r < RK_RPW; ++r) acc[r][p] += w[r].x * e[p].x + w[r].y * e[p].y + w[r].z * e[p].z + w[r].w * e[p].w;
  }
#pragma unroll
  for (int r = 0; r < RK_RPW; ++r)
#pragma unroll
    for (int p = 0; p < RK_PB; ++p) {
      const float v = wave_sum(acc[r][p]);
      if (lane == 0 && g0 + r < G && p0 + p < P) scores[(size_t)(p0 + p) * G + g0 + r] = v;
    }
}

// order-preserving map of a float's bits: larger float <=> larger unsigned key (-0 counts as +0)
__device__ __forceinline__ uint32_t score_key(float f) {
  const uint32_t u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exact top-K of one prompt's G scores.  One workgroup of 1024 lanes per prompt, keys in LDS.  Four radix passes
// (8 bits each, from the top) find the K-th largest key T; the selected set is {key > T} plus the lowest-id
// members of {key == T} up to K; ids come out ascending through a block prefix sum in id order.
__global__ __launch_bounds__(1024) void rank_topk(const float *__restrict__ scores, int G, int K,
                                                  int32_t *__restrict__ subset_out, int subset_stride) {
  __shared__ uint32_t keys[RK_MAXG];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sel_prefix, sel_need;
  __shared__ int32_t scan_gt[1024], scan_eq[1024];
  const int p = blockIdx.x, tid = threadIdx.x;
  for (int g = tid; g < G; g += 1024) keys[g] = score_key(scores[(size_t)p * G + g]);
  if (tid == 0) { sel_prefix = 0u; sel_need = (uint32_t)K; }
  __syncthreads();
  // after the pass for byte b, sel_prefix holds the top bytes of T and sel_need the number still to take among
  // the keys that share them
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0u;
    __syncthreads();
    const uint32_t prefix = sel_prefix;
    const uint32_t himask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (int g = tid; g < G; g += 1024) {
      const uint32_t kx = keys[g];
      if ((kx & himask) == (prefix & himask)) atomicAdd(&hist[(kx >> shift) & 0xFFu], 1u);
    }
    __syncthreads();
    // suffix sums over the 256 bins (Hillis-Steele, in place): hist[b] = keys with byte >= b; the wanted bin is
    // the one whose suffix reaches `need` while the next one does not
    for (int o = 1; o < 256; o <<= 1) {
      const uint32_t add = (tid < 256 && tid + o < 256) ? hist[tid + o] : 0u;
      __syncthreads();
      if (tid < 256) hist[tid] += add;
      __syncthreads();
    }
    const uint32_t need = sel_need;
    __syncthreads();
    if (tid < 256) {
      const uint32_t here = hist[tid], above = tid < 255 ? hist[tid + 1] : 0u;
      if (here >= need && above < need) {          // exactly one bin (the total is >= need by construction)
        sel_prefix = prefix | ((uint32_t)tid << shift);
        sel_need = need - above;
      }
    }
    __syncthreads();
  }
  const uint32_t T = sel_prefix;
  const int need_eq = (int)sel_need;             // members of {key == T} to take, lowest ids first
  // ids in contiguous segments per lane, counts scanned over the block in id order
  const int per = (G + 1023) / 1024;
  const int s0 = min(tid * per, G), s1 = min(s0 + per, G);
  int ngt = 0, neq = 0;
  for (int g = s0; g < s1; ++g) { ngt += keys[g] > T ? 1 : 0; neq += keys[g] == T ? 1 : 0; }
  scan_gt[tid] = ngt; scan_eq[tid] = neq;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    const int a = tid >= o ? scan_gt[tid - o] : 0, b = tid >= o ? scan_eq[tid - o] : 0;
    __syncthreads();
    scan_gt[tid] += a; scan_eq[tid] += b;
    __syncthreads();
  }
  int before_gt = scan_gt[tid] - ngt, before_eq = scan_eq[tid] - neq;   // exclusive
  for (int g = s0; g < s1; ++g) {
    const uint32_t kx = keys[g];
    const bool eq = kx == T;
    const bool take = kx > T || (eq && before_eq < need_eq);
    if (take) {
      const int pos = before_gt + min(before_eq, need_eq);
      if (pos < K) subset_out[(size_t)p * subset_stride + pos] = g;
    }
    before_gt += kx > T ? 1 : 0;
    before_eq += eq ? 1 : 0;
  }
}

// Gather + reorder.  One thread per 16-byte output piece of the operand-order blocks (index maps as in the
// offline reorder); rank r of pattern j is row subset[j*stride + r] of the row-major layer.  Out-of-range ids
// give zero rows.
__global__ void gather_mfma16_v(const uint16_t *__restrict__ Vt, int R, int n, const int32_t *__restrict__ subset,
                                int stride, int K, uint16_t *__restrict__ dst) {
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t per_pattern = (size_t)K * n / 8;
  if (o >= per_pattern) return;
  const int pat = blockIdx.y;
  const int j = o & 31, q = (o >> 5) & 1;
  const size_t t = o >> 6;
  const int kb = t % (n / 16), rb = t / (n / 16);
  const int row = subset[(size_t)pat * stride + rb * 32 + j];
  u32x4 v = {0, 0, 0, 0};
  if (row >= 0 && row < R) v = *reinterpret_cast<const u32x4 *>(Vt + (size_t)row * n + kb * 16 + q * 8);
  *reinterpret_cast<u32x4 *>(dst + ((size_t)pat * per_pattern + o) * 8) = v;
}

__global__ void gather_mfma16_u(const uint16_t *__restrict__ Ut, int R, int m, const int32_t *__restrict__ subset,
                                int stride, int K, uint16_t *__restrict__ dst) {
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t per_pattern = (size_t)K * m / 8;
  if (o >= per_pattern) return;
  const int pat = blockIdx.y;
  const int j = o & 31, q = (o >> 5) & 1;
  const size_t t = o >> 6;
  const int cb = t % (m / 32), kb = t / (m / 32);
  const int c = cb * 32 + j, r0 = kb * 16 + q * 8;
  uint16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int row = subset[(size_t)pat * stride + r0 + e];
    v[e] = (row >= 0 && row < R) ? Ut[(size_t)row * m + c] : (uint16_t)0;
  }
  u32x4 w;
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = (uint32_t)v[2 * e] | ((uint32_t)v[2 * e + 1] << 16);
  *reinterpret_cast<u32x4 *>(dst + ((size_t)pat * per_pattern + o) * 8) = w;
}

}  // namespace parse

using namespace parse;

extern "C" {

size_t parse_route_ranks_workspace_bytes(int32_t rows, int32_t P, int32_t d, int32_t G) {
  if (rows <= 0 || P <= 0 || d <= 0 || G <= 0) return 0;
  // pooling partials (as the grouped router), embeddings, scores
  return parse_route_workspace_bytes(rows, P, d) + round_up((size_t)P * d * sizeof(float), 256) +
         round_up((size_t)P * G * sizeof(float), 256);
}

int parse_route_ranks(const void *X, int32_t xdtype, int32_t rows, const int32_t *tok_offsets, int32_t P, int32_t d,
                      const float *Wr, int32_t G, int32_t K, int32_t *subset_out, int32_t subset_stride,
                      float *scores_out, float *emb_out, void *workspace, size_t workspace_bytes,
                      parse_stream stream) {
  if (!X || !tok_offsets || !Wr || !subset_out) return PARSE_EINVAL;
  if (xdtype != PARSE_F32 && xdtype != PARSE_BF16) return PARSE_EINVAL;
  if (rows <= 0 || P <= 0 || d <= 0 || G <= 0 || K <= 0) return PARSE_EINVAL;
  if (K > G || G > RK_MAXG || d > 16384 || P > rows || P > 65535 || subset_stride < K) return PARSE_ESHAPE;
  if (d % 8 != 0) return PARSE_EALIGN;
  if (!aligned16(X) || !aligned16(Wr) || !aligned16(workspace)) return PARSE_EALIGN;
  if ((emb_out && !aligned16(emb_out)) || (scores_out && !aligned16(scores_out))) return PARSE_EALIGN;
  if (!workspace || workspace_bytes < parse_route_ranks_workspace_bytes(rows, P, d, G)) return PARSE_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char *ws = reinterpret_cast<char *>(workspace);
  const size_t pool_bytes = parse_route_workspace_bytes(rows, P, d);
  float *partial = reinterpret_cast<float *>(ws);
  float *emb = emb_out ? emb_out : reinterpret_cast<float *>(ws + pool_bytes);
  float *scores = scores_out ? scores_out
                             : reinterpret_cast<float *>(ws + pool_bytes + round_up((size_t)P * d * sizeof(float), 256));
  int Q = 0;
  int st = launch_pool_partials(X, xdtype, rows, tok_offsets, P, d, partial, &Q, s);
  if (st != PARSE_OK) return st;
  st = launch_pool_finish(partial, Q, rows, d, tok_offsets, P, emb, s);
  if (st != PARSE_OK) return st;
  hipLaunchKernelGGL(rank_scores, dim3((G + RK_ROWS - 1) / RK_ROWS, (P + RK_PB - 1) / RK_PB), dim3(256), 0, s, Wr, emb, G,
                     d, P, scores);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(rank_topk, dim3(P), dim3(1024), 0, s, scores, G, K, subset_out, subset_stride);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

int parse_pack_ranks(const parse_layer *L, const int32_t *subset, int32_t subset_stride, int32_t K,
                     int32_t n_patterns, void *Vt_S, void *Ut_S, parse_stream stream) {
  int st = check_layer(L);
  if (st != PARSE_OK) return st;
  if (!subset || !Vt_S || !Ut_S) return PARSE_EINVAL;
  if (K <= 0 || n_patterns <= 0) return PARSE_EINVAL;
  if (L->dtype != PARSE_BF16 || L->layout != PARSE_ROWMAJOR) return PARSE_ELAYOUT;
  if (K % 32 != 0 || L->n % 16 != 0 || L->m % 32 != 0 || subset_stride < K || n_patterns > 65535) return PARSE_ESHAPE;
  if (!aligned16(Vt_S) || !aligned16(Ut_S)) return PARSE_EALIGN;
  hipStream_t s = (hipStream_t)stream;
  const size_t nv = (size_t)K * L->n / 8, nu = (size_t)K * L->m / 8;
  hipLaunchKernelGGL(gather_mfma16_v, dim3((unsigned)((nv + 255) / 256), n_patterns), dim3(256), 0, s,
                     (const uint16_t *)L->Vt, L->R, L->n, subset, subset_stride, K, (uint16_t *)Vt_S);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(gather_mfma16_u, dim3((unsigned)((nu + 255) / 256), n_patterns), dim3(256), 0, s,
                     (const uint16_t *)L->Ut, L->R, L->m, subset, subset_stride, K, (uint16_t *)Ut_S);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // extern "C"
