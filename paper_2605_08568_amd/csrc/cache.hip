// a3: pattern cache (Sec. 4.3, "Rank Retrieval for Prefilling"): prompt embedding -> rank subsets of all
// L routed matrices, answered by the nearest stored key under cosine similarity.
//
// Kernels of one batched probe (all on the caller's stream, no host round trip; the entry count lives
// in device memory):
//   cache_sims       cosine of every prompt with every stored key and, for the sequential variant, with
//                    every earlier prompt of the batch; one wavefront per (prompt, column), norms on the fly
//   resolve          one workgroup: its wavefronts first take the arg-max over the stored keys per prompt
//                    (smallest index on ties), then ONE wavefront walks the batch in arrival order and
//                    decides hit / miss / new entry, taking earlier misses of the same batch (already
//                    appended) into account
//   route_or_gather  per (layer, prompt): a miss runs the router (scores + top-k) and appends key and
//                    subsets; a hit on a stored entry copies its subsets; a hit on an entry appended by
//                    this very batch re-routes that entry's key (same result as the stored value, which
//                    another workgroup of this launch is still writing)
#include <new>

#include "common.hpp"
#include "topk.hpp"

struct parse_cache {
  int32_t capacity, d, L, k, max_batch;
  float *keys;      // [capacity][d]
  int32_t *values;  // [capacity][L][k]
  int32_t *count;   // [3]: the live counter is count[cur] (cur = 0/1; a fused probe reads it and writes the other one);
                    //      count[2] = explicit inserts dropped because the cache was full
  int32_t cur;
  // scratch of one batch
  float *sims;      // [max_batch][capacity + max_batch]
  int32_t *src;     // [max_batch] prompt whose embedding defines the answer's key (in-batch entries), else -1
  int32_t *entry;   // [max_batch] (used when the caller passes no entry_out)
  uint8_t *hit;     // [max_batch]
  int32_t n_shared; // leading groups every routed subset holds (route-on-miss uses it)
  int32_t count_ub; // host-side upper bound of *count (exact after count and clear); sizes the probe grid
};

namespace parse {

// grid (ceil((ncols_keys + peers)/4), P), block 256: wave w of block bx handles column j = 4*bx + w.
// Columns [0, ncols_keys) are stored keys (skipped beyond *count), the next `peers` columns are batch peers
// (only q < p is needed); similarities land in sims[p][j] (keys) and sims[p][capacity + q] (peers).
__global__ __launch_bounds__(256) void cache_sims(const float *__restrict__ E, int d, const float *__restrict__ keys,
                                                  const int32_t *__restrict__ count, int capacity, int ncols_keys,
                                                  int peers, int ld, float *__restrict__ sims) {
  const int p = blockIdx.y, lane = threadIdx.x & 63;
  int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  const float *other;
  if (j < ncols_keys) {
    if (j >= *count || j >= capacity) return;
    other = keys + (size_t)j * d;
  } else {
    const int q = j - ncols_keys;
    j = capacity + q;
    if (q >= peers || q >= p) return;
    other = E + (size_t)q * d;
  }
  const float4 *a4 = reinterpret_cast<const float4 *>(E + (size_t)p * d);
  const float4 *b4 = reinterpret_cast<const float4 *>(other);
  float ab = 0.f, aa = 0.f, bb = 0.f;
#pragma unroll 8
  for (int c = lane; c < d / 4; c += 64) {
    const float4 a = a4[c], b = b4[c];
    ab += a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
    aa += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
    bb += b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
  }
  ab = wave_sum(ab); aa = wave_sum(aa); bb = wave_sum(bb);
  if (lane == 0) sims[(size_t)p * ld + j] = ab / (sqrtf(aa) * sqrtf(bb));
}

__device__ __forceinline__ void wave_argmax(float &bs, int &bi) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float os = __shfl_xor(bs, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    const bool take = (oi >= 0) && (bi < 0 || os > bs || (os == bs && oi < bi));
    if (take) { bs = os; bi = oi; }
  }
}

// One workgroup of 1024 lanes.  LDS: best_sim[P], best_idx[P], ins_list[P].
// sequential == 0: pure lookup (threshold the best stored key).  Otherwise arrival-order semantics: ins_list
// holds the prompts appended so far in this batch; the i-th of them became entry count0 + i.
__global__ __launch_bounds__(1024) void resolve(const float *__restrict__ sims, int ld, int capacity, int P,
                                                float tau, int sequential, int32_t *__restrict__ count,
                                                int32_t *__restrict__ entry_out, uint8_t *__restrict__ hit_out,
                                                float *__restrict__ sim_out, int32_t *__restrict__ src_out) {
  extern __shared__ float lds_f[];
  float *best_sim = lds_f;                                         // [P]
  int32_t *best_idx = reinterpret_cast<int32_t *>(lds_f + P);      // [P]
  int32_t *ins_list = best_idx + P;                                // [P]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int count0 = *count;
  for (int p = wave; p < P; p += nwaves) {
    float bs = -INFINITY;
    int bi = -1;
    for (int j = lane; j < count0; j += 64) {
      const float s = sims[(size_t)p * ld + j];
      if (bi < 0 || s > bs) { bs = s; bi = j; }
    }
    wave_argmax(bs, bi);
    if (lane == 0) { best_sim[p] = bs; best_idx[p] = bi; }
  }
  __syncthreads();
  if (!sequential) {
    for (int p = threadIdx.x; p < P; p += blockDim.x) {
      const bool h = best_idx[p] >= 0 && best_sim[p] >= tau;
      entry_out[p] = h ? best_idx[p] : -1;
      hit_out[p] = h ? 1 : 0;
      src_out[p] = -1;
      if (sim_out) sim_out[p] = best_sim[p];
    }
    return;
  }
  if (wave != 0) return;
  int n_ins = 0;
  for (int p = 0; p < P; ++p) {
    float bs = best_sim[p];
    int bi = best_idx[p];
    // best among the peers appended so far: larger similarity wins, equal similarity keeps the lower entry
    float ps = -INFINITY;
    int pi = -1;
    for (int i = lane; i < n_ins; i += 64) {
      const float s = sims[(size_t)p * ld + capacity + ins_list[i]];
      if (pi < 0 || s > ps) { ps = s; pi = i; }
    }
    wave_argmax(ps, pi);
    int src = -1;
    if (pi >= 0 && (bi < 0 || ps > bs)) { bs = ps; bi = count0 + pi; src = ins_list[pi]; }
    const bool h = bi >= 0 && bs >= tau;
    int ent;
    if (h) {
      ent = bi;
    } else if (count0 + n_ins < capacity) {
      ent = count0 + n_ins;
      if (lane == 0) ins_list[n_ins] = p;
      ++n_ins;
    } else {
      ent = -1;
    }
    __builtin_amdgcn_s_waitcnt(0);  // the ins_list write is visible to this wave's later reads
    __builtin_amdgcn_wave_barrier();
    if (lane == 0) {
      entry_out[p] = ent;
      hit_out[p] = h ? 1 : 0;
      src_out[p] = h ? src : -1;
      if (sim_out) sim_out[p] = bs;
    }
  }
  if (lane == 0) *count = count0 + n_ins;
}

// grid (L, P), block 256, LDS d + 128 floats.  do_route == 0 (pure lookup): only the copy for hits.
__global__ __launch_bounds__(256) void route_or_gather(const float *__restrict__ E, int d, const float *__restrict__ Wr,
                                                       int G, int L, int k, int capacity, int do_route,
                                                       const int32_t *__restrict__ entry, const uint8_t *__restrict__ hit,
                                                       const int32_t *__restrict__ src, float *__restrict__ keys,
                                                       int32_t *__restrict__ values, int32_t *__restrict__ subset_out,
                                                       int n_shared) {
  extern __shared__ float lds[];
  float *e = lds, *s = lds + d;
  const int l = blockIdx.x, p = blockIdx.y;
  const int ent = entry[p];
  const bool h = hit[p] != 0;
  if (h && src[p] < 0) {          // answered by an entry stored before this batch
    if (ent >= 0 && ent < capacity && threadIdx.x < k)
      subset_out[((size_t)p * L + l) * k + threadIdx.x] = values[((size_t)ent * L + l) * k + threadIdx.x];
    return;
  }
  if (!do_route) return;
  const int from = h ? src[p] : p;  // the embedding that defines the key of the answering entry
  const bool owner = !h && ent >= 0;   // this prompt's miss created entry `ent`
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = E[(size_t)from * d + c];
    e[c] = v;
    if (l == 0 && owner) keys[(size_t)ent * d + c] = v;
  }
  __syncthreads();
  block_router_scores(Wr + (size_t)l * G * d, e, d, G, s);
  int32_t *sel = reinterpret_cast<int32_t *>(s + 64);  // [64] after the scores
  if (threadIdx.x < 64) wave_topk_ascending(s, G, k, sel, n_shared);
  __syncthreads();
  if (threadIdx.x < k) {
    const int32_t g = sel[threadIdx.x];
    subset_out[((size_t)p * L + l) * k + threadIdx.x] = g;
    if (owner) values[((size_t)ent * L + l) * k + threadIdx.x] = g;
  }
}

// Small batches (P <= kSmallBatch): resolve and route_or_gather in one launch.  grid (L, P), block 256.  Every
// workgroup repeats the (cheap, deterministic) decision walk for prompts 0..p from the similarity matrix, so no
// workgroup waits for another; it then routes / gathers for its own (layer, prompt).  The entry count is read
// from count_in and the new one written to count_out (a different word: workgroups still starting must see the
// old value) by the workgroup of the last prompt, which has walked the whole batch.
constexpr int kSmallBatch = 64;
__global__ __launch_bounds__(256) void resolve_route_or_gather(
    const float *__restrict__ sims, int ld, int capacity, int P, float tau, const int32_t *__restrict__ count_in,
    int32_t *__restrict__ count_out, const float *__restrict__ E, int d, const float *__restrict__ Wr, int G, int L, int k,
    int32_t *__restrict__ entry_out, uint8_t *__restrict__ hit_out, float *__restrict__ sim_out,
    float *__restrict__ keys, int32_t *__restrict__ values, int32_t *__restrict__ subset_out, int n_shared) {
  extern __shared__ float lds[];
  float *e = lds, *s = lds + d;
  __shared__ float best_sim[kSmallBatch];
  __shared__ int32_t best_idx[kSmallBatch], ins_list[kSmallBatch];
  __shared__ int32_t my_ent, my_src, my_hit, total_ins;
  __shared__ float peer[kSmallBatch][kSmallBatch + 1];   // peer[q][i] = similarity of prompt q with earlier prompt i
  const int l = blockIdx.x, p = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int count0 = min(*count_in, capacity);
  // the walk below is sequential: everything it reads is fetched here, all at once
  for (int t = threadIdx.x; t < (p + 1) * P; t += blockDim.x) {
    const int q = t / P, i = t - q * P;
    if (i < q) peer[q][i] = sims[(size_t)q * ld + capacity + i];
  }
  for (int q = wave; q <= p; q += nwaves) {
    float bs = -INFINITY;
    int bi = -1;
    for (int j = lane; j < count0; j += 64) {
      const float v = sims[(size_t)q * ld + j];
      if (bi < 0 || v > bs) { bs = v; bi = j; }
    }
    wave_argmax(bs, bi);
    if (lane == 0) { best_sim[q] = bs; best_idx[q] = bi; }
  }
  __syncthreads();
  if (wave == 0) {
    int n_ins = 0;
    for (int q = 0; q <= p; ++q) {
      float bs = best_sim[q];
      int bi = best_idx[q];
      // best among the peers appended so far: larger similarity wins, equal similarity keeps the lower entry
      float ps = -INFINITY;
      int pi = -1;
      for (int i = lane; i < n_ins; i += 64) {
        const float v = peer[q][ins_list[i]];
        if (pi < 0 || v > ps) { ps = v; pi = i; }
      }
      wave_argmax(ps, pi);
      int src = -1;
      if (pi >= 0 && (bi < 0 || ps > bs)) { bs = ps; bi = count0 + pi; src = ins_list[pi]; }
      const bool h = bi >= 0 && bs >= tau;
      int ent;
      if (h) {
        ent = bi;
      } else if (count0 + n_ins < capacity) {
        ent = count0 + n_ins;
        if (lane == 0) ins_list[n_ins] = q;
        ++n_ins;
      } else {
        ent = -1;
      }
      __builtin_amdgcn_s_waitcnt(0);  // the ins_list write is visible to this wave's later reads
      __builtin_amdgcn_wave_barrier();
      if (q == p && lane == 0) {
        my_ent = ent; my_hit = h ? 1 : 0; my_src = h ? src : -1;
        if (l == 0) {
          entry_out[p] = ent;
          hit_out[p] = h ? 1 : 0;
          if (sim_out) sim_out[p] = bs;
        }
      }
    }
    if (lane == 0) total_ins = n_ins;
  }
  __syncthreads();
  if (l == 0 && p == P - 1 && threadIdx.x == 0) *count_out = count0 + total_ins;
  const int ent = my_ent;
  const bool h = my_hit != 0;
  if (h && my_src < 0) {          // answered by an entry stored before this batch
    if (ent >= 0 && ent < capacity && (int)threadIdx.x < k)
      subset_out[((size_t)p * L + l) * k + threadIdx.x] = values[((size_t)ent * L + l) * k + threadIdx.x];
    return;
  }
  const int from = h ? my_src : p;     // the embedding that defines the key of the answering entry
  const bool owner = !h && ent >= 0;   // this prompt's miss created entry `ent`
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = E[(size_t)from * d + c];
    e[c] = v;
    if (l == 0 && owner) keys[(size_t)ent * d + c] = v;
  }
  __syncthreads();
  block_router_scores(Wr + (size_t)l * G * d, e, d, G, s);
  int32_t *sel = reinterpret_cast<int32_t *>(s + 64);  // [64] after the scores
  if (threadIdx.x < 64) wave_topk_ascending(s, G, k, sel, n_shared);
  __syncthreads();
  if ((int)threadIdx.x < k) {
    const int32_t g = sel[threadIdx.x];
    subset_out[((size_t)p * L + l) * k + threadIdx.x] = g;
    if (owner) values[((size_t)ent * L + l) * k + threadIdx.x] = g;
  }
}

__global__ void append_entry(const float *__restrict__ emb, const int32_t *__restrict__ subsets, int d, int Lk,
                             int32_t *__restrict__ count, int32_t *__restrict__ dropped, int capacity,
                             float *__restrict__ keys, int32_t *__restrict__ values) {
  const int ent = *count;
  if (ent >= capacity) {               // full: the entry is dropped and counted (one workgroup: no race)
    if (threadIdx.x == 0) *dropped += 1;
    return;
  }
  for (int c = threadIdx.x; c < d; c += blockDim.x) keys[(size_t)ent * d + c] = emb[c];
  for (int i = threadIdx.x; i < Lk; i += blockDim.x) values[(size_t)ent * Lk + i] = subsets[i];
  __syncthreads();   // one workgroup: every lane has read *count before it changes
  if (threadIdx.x == 0) *count = ent + 1;
}

__global__ void set_i32(int32_t *p, int32_t v) { *p = v; }

static int check_probe(const parse_cache *c, const float *emb, int P) {
  if (!c || !emb) return PARSE_EINVAL;
  if (P <= 0) return PARSE_EINVAL;
  if (P > c->max_batch) return PARSE_ESHAPE;
  if (!aligned16(emb)) return PARSE_EALIGN;
  return PARSE_OK;
}

}  // namespace parse

using namespace parse;

extern "C" {

int parse_cache_create(parse_cache **out, int32_t capacity, int32_t d, int32_t L, int32_t k, int32_t max_batch) {
  if (!out) return PARSE_EINVAL;
  *out = nullptr;
  if (capacity <= 0 || d <= 0 || L <= 0 || k <= 0 || max_batch <= 0) return PARSE_EINVAL;
  if (d % 4 != 0) return PARSE_EALIGN;
  if (d > 16384 || k > 64 || max_batch > 4096) return PARSE_ESHAPE;
  parse_cache *c = new (std::nothrow) parse_cache();
  if (!c) return PARSE_EINVAL;
  c->capacity = capacity; c->d = d; c->L = L; c->k = k; c->max_batch = max_batch;
  c->count_ub = 0;
  c->cur = 0;
  c->n_shared = 0;
  const size_t ld = (size_t)capacity + max_batch;
  hipError_t e = hipSuccess;
  auto alloc = [&](void **p, size_t bytes) {
    if (e == hipSuccess) e = hipMalloc(p, round_up(bytes, 256));
  };
  alloc((void **)&c->keys, (size_t)capacity * d * sizeof(float));
  alloc((void **)&c->values, (size_t)capacity * L * k * sizeof(int32_t));
  alloc((void **)&c->count, 4 * sizeof(int32_t));
  alloc((void **)&c->sims, (size_t)max_batch * ld * sizeof(float));
  alloc((void **)&c->src, (size_t)max_batch * sizeof(int32_t));
  alloc((void **)&c->entry, (size_t)max_batch * sizeof(int32_t));
  alloc((void **)&c->hit, (size_t)max_batch);
  if (e == hipSuccess) e = hipMemset(c->count, 0, 4 * sizeof(int32_t));
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    set_hip_error(e, "parse_cache_create");
    parse_cache_destroy(c);
    return PARSE_EHIP;
  }
  *out = c;
  return PARSE_OK;
}

int parse_cache_destroy(parse_cache *c) {
  if (!c) return PARSE_EINVAL;
  (void)hipDeviceSynchronize();
  void *ptrs[] = {c->keys, c->values, c->count, c->sims, c->src, c->entry, c->hit};
  for (void *p : ptrs)
    if (p) (void)hipFree(p);
  delete c;
  return PARSE_OK;
}

int parse_cache_set_shared(parse_cache *c, int32_t n_shared) {
  if (!c || n_shared < 0) return PARSE_EINVAL;
  if (n_shared > c->k) return PARSE_ESHAPE;
  c->n_shared = n_shared;
  return PARSE_OK;
}

int parse_cache_clear(parse_cache *c, parse_stream stream) {
  if (!c) return PARSE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(set_i32, dim3(1), dim3(1), 0, s, c->count + c->cur, 0);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(set_i32, dim3(1), dim3(1), 0, s, c->count + 2, 0);
  PARSE_LAUNCH_CHECK();
  c->count_ub = 0;     // exact again: every later call on the cache is ordered after the two stores
  return PARSE_OK;
}

int parse_cache_count(parse_cache *c, int32_t *count_out, int32_t *dropped_out, parse_stream stream) {
  if (!c || !count_out) return PARSE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  int32_t both[2] = {0, 0};
  PARSE_HIP_TRY(hipMemcpyAsync(&both[0], c->count + c->cur, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  PARSE_HIP_TRY(hipMemcpyAsync(&both[1], c->count + 2, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  PARSE_HIP_TRY(hipStreamSynchronize(s));
  *count_out = both[0];
  if (dropped_out) *dropped_out = both[1];
  c->count_ub = both[0];
  return PARSE_OK;
}

int parse_cache_insert(parse_cache *c, const float *emb, const int32_t *subsets, parse_stream stream) {
  if (!c || !emb || !subsets) return PARSE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(append_entry, dim3(1), dim3(256), 0, s, emb, subsets, c->d, c->L * c->k, c->count + c->cur, c->count + 2,
                     c->capacity, c->keys, c->values);
  PARSE_LAUNCH_CHECK();
  c->count_ub = c->count_ub + 1 < c->capacity ? c->count_ub + 1 : c->capacity;
  return PARSE_OK;
}

int parse_cache_lookup(parse_cache *c, const float *emb, int32_t P, float tau, int32_t *entry_out, float *sim_out,
                       int32_t *subset_out, parse_stream stream) {
  int st = check_probe(c, emb, P);
  if (st != PARSE_OK) return st;
  if (!entry_out) return PARSE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const int ld = c->capacity + c->max_batch;
  const int ncols = c->count_ub < c->capacity ? c->count_ub : c->capacity;
  if (ncols > 0) {
    hipLaunchKernelGGL(cache_sims, dim3((ncols + 3) / 4, P), dim3(256), 0, s, emb, c->d, c->keys, c->count + c->cur, c->capacity,
                       ncols, 0, ld, c->sims);
    PARSE_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(resolve, dim3(1), dim3(1024), (size_t)P * 12, s, c->sims, ld, c->capacity, P, tau, 0, c->count + c->cur,
                     entry_out, c->hit, sim_out, c->src);
  PARSE_LAUNCH_CHECK();
  if (subset_out) {
    hipLaunchKernelGGL(route_or_gather, dim3(c->L, P), dim3(256), 0, s, emb, c->d, (const float *)nullptr, 0, c->L,
                       c->k, c->capacity, 0, entry_out, c->hit, c->src, c->keys, c->values, subset_out, 0);
    PARSE_LAUNCH_CHECK();
  }
  return PARSE_OK;
}

int parse_cache_lookup_or_route(parse_cache *c, const float *emb, int32_t P, float tau, const float *Wr, int32_t G,
                                int32_t *entry_out, uint8_t *hit_out, float *sim_out, int32_t *subset_out,
                                parse_stream stream) {
  int st = check_probe(c, emb, P);
  if (st != PARSE_OK) return st;
  if (!Wr || !subset_out) return PARSE_EINVAL;
  if (G <= 0) return PARSE_EINVAL;
  if (G > 64 || c->k > G) return PARSE_ESHAPE;
  if (!aligned16(Wr)) return PARSE_EALIGN;
  hipStream_t s = (hipStream_t)stream;
  const int ld = c->capacity + c->max_batch;
  int32_t *entry = entry_out ? entry_out : c->entry;
  uint8_t *hit = hit_out ? hit_out : c->hit;
  const int ncols = c->count_ub < c->capacity ? c->count_ub : c->capacity;
  if (ncols + P > 1) {   // a single prompt against an empty cache has nothing to compare with
    hipLaunchKernelGGL(cache_sims, dim3((ncols + P + 3) / 4, P), dim3(256), 0, s, emb, c->d, c->keys, c->count + c->cur,
                       c->capacity, ncols, P, ld, c->sims);
    PARSE_LAUNCH_CHECK();
  }
  c->count_ub = (c->count_ub + P < c->capacity) ? c->count_ub + P : c->capacity;
  if (P <= kSmallBatch) {
    // small batch: every (layer, prompt) workgroup works out the batch's decisions itself, then does its own part;
    // the new entry count goes to the other counter slot, which becomes the live one
    PARSE_ALLOW_LDS(resolve_route_or_gather, (size_t)(c->d + 128) * sizeof(float));
    hipLaunchKernelGGL(resolve_route_or_gather, dim3(c->L, P), dim3(256), (size_t)(c->d + 128) * sizeof(float), s, c->sims,
                       ld, c->capacity, P, tau, c->count + c->cur, c->count + (c->cur ^ 1), emb, c->d, Wr, G, c->L, c->k,
                       entry, hit, sim_out, c->keys, c->values, subset_out, c->n_shared);
    PARSE_LAUNCH_CHECK();
    c->cur ^= 1;
    return PARSE_OK;
  }
  hipLaunchKernelGGL(resolve, dim3(1), dim3(1024), (size_t)P * 12, s, c->sims, ld, c->capacity, P, tau, 1, c->count + c->cur,
                     entry, hit, sim_out, c->src);
  PARSE_LAUNCH_CHECK();
  PARSE_ALLOW_LDS(route_or_gather, (size_t)(c->d + 128) * sizeof(float));
  hipLaunchKernelGGL(route_or_gather, dim3(c->L, P), dim3(256), (size_t)(c->d + 128) * sizeof(float), s, emb, c->d, Wr,
                     G, c->L, c->k, c->capacity, 1, entry, hit, c->src, c->keys, c->values, subset_out, c->n_shared);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // extern "C"
