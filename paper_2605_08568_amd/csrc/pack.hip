// a4: expert memory aggregation (Sec. 4.4) and the offline reorder into matrix-core operand order.
//
//   pack_slabs        every selected rank group is one contiguous slab in both factor matrices (in either
//                     layout), so aggregation is 2k slab copies: 16 bytes per lane, 1 KiB per wavefront
//                     instruction, read once / written once.
//   to_mfma16_v / _u  row-major bf16 -> PARSE_MFMA16 order (index maps documented in parse.h).
#include "common.hpp"

namespace parse {

constexpr int kCopyThreads = 256;
constexpr int kCopyUnroll = 8;                                       // 16-byte pieces per lane per block
constexpr size_t kCopyChunk = (size_t)kCopyThreads * kCopyUnroll * 16;  // 32 KiB per block

constexpr int kPackWindow = 2048;   // patterns whose work list a workgroup holds in LDS at a time

// A fixed grid walks the work list: every workgroup first lists (in LDS) the patterns that have anything to
// copy -- a batch whose prompts all hit the cache ends here, after one pass over the hit flags -- then takes
// every gridDim.x-th task; a task = (listed pattern, one of its 2k slabs, one 32 KiB chunk of the slab).
// The list is in ascending pattern order in every workgroup (a strided walk over lists that differ from
// workgroup to workgroup would copy some tasks twice and others never).
__global__ __launch_bounds__(kCopyThreads) void pack_slabs(const char *__restrict__ Vt, const char *__restrict__ Ut,
                                                           size_t v_slab_bytes, size_t u_slab_bytes, int G, int k,
                                                           const int32_t *__restrict__ subset, int subset_stride,
                                                           const int32_t *__restrict__ rep,
                                                           const int32_t *__restrict__ slot,
                                                           const uint8_t *__restrict__ skip, int n_slots,
                                                           const int32_t *__restrict__ n_patterns, int max_patterns,
                                                           char *__restrict__ Vt_S, char *__restrict__ Ut_S) {
  __shared__ int32_t act[kPackWindow];
  __shared__ int32_t n_act;
  __shared__ int32_t wave_cnt[kCopyThreads / 64];
  const int np = n_patterns ? min(*n_patterns, max_patterns) : max_patterns;
  const size_t big = v_slab_bytes > u_slab_bytes ? v_slab_bytes : u_slab_bytes;
  const int chunks = (int)((big + kCopyChunk - 1) / kCopyChunk);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int j0 = 0; j0 < np; j0 += kPackWindow) {
    if (threadIdx.x == 0) n_act = 0;
    __syncthreads();
    // the list is filled in ascending pattern order (per-wavefront vote + prefix over the wavefronts), so every
    // workgroup holds the SAME list and the strided walk below covers every task exactly once
    const int wend = min(np, j0 + kPackWindow);
    for (int r0 = j0; r0 < wend; r0 += kCopyThreads) {
      const int j = r0 + (int)threadIdx.x;
      bool on = j < wend && !(skip && skip[j]);
      if (on && rep) on = rep[j] >= 0;
      if (on) {
        const int d = slot ? slot[j] : j;
        on = d >= 0 && d < n_slots;
      }
      const unsigned long long votes = __ballot(on);
      if (lane == 0) wave_cnt[wave] = __popcll(votes);
      __syncthreads();
      int base = n_act;
      for (int w2 = 0; w2 < wave; ++w2) base += wave_cnt[w2];
      if (on) act[base + __popcll(votes & ((1ull << lane) - 1ull))] = j;
      __syncthreads();
      if (threadIdx.x == 0) {
        int add = 0;
        for (int w2 = 0; w2 < kCopyThreads / 64; ++w2) add += wave_cnt[w2];
        n_act += add;
      }
      __syncthreads();
    }
    const long long total = (long long)n_act * 2 * k * chunks;
    for (long long t = blockIdx.x; t < total; t += gridDim.x) {
      const int c = (int)(t % chunks);
      const int y = (int)((t / chunks) % (2 * k));
      const int j = act[t / ((long long)chunks * 2 * k)];
      const int row = rep ? rep[j] : j;
      const int dst_slot = slot ? slot[j] : j;
      const bool is_u = y >= k;
      const int slot_in = is_u ? y - k : y;
      const int g = subset[(size_t)row * subset_stride + slot_in];
      if (g < 0 || g >= G) continue;
      const size_t slab = is_u ? u_slab_bytes : v_slab_bytes;
      const size_t base = (size_t)c * kCopyChunk;
      if (base >= slab) continue;
      const char *src = (is_u ? Ut : Vt) + (size_t)g * slab;
      char *dst = (is_u ? Ut_S : Vt_S) + ((size_t)dst_slot * k + slot_in) * slab;
      u32x4 v[kCopyUnroll];
#pragma unroll
      for (int i = 0; i < kCopyUnroll; ++i) {
        const size_t o = base + ((size_t)i * kCopyThreads + threadIdx.x) * 16;
        if (o < slab) v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
      }
#pragma unroll
      for (int i = 0; i < kCopyUnroll; ++i) {
        const size_t o = base + ((size_t)i * kCopyThreads + threadIdx.x) * 16;
        if (o < slab) *reinterpret_cast<u32x4 *>(dst + o) = v[i];
      }
    }
    __syncthreads();
  }
}

// One thread per 16-byte output piece.  Output piece index o = ((rb*(n/16) + kb)*2 + q)*32 + j.
__global__ void to_mfma16_v(const uint16_t *__restrict__ src, int R, int n, uint16_t *__restrict__ dst) {
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = (size_t)R * n / 8;
  if (o >= total) return;
  const int j = o & 31, q = (o >> 5) & 1;
  const size_t t = o >> 6;
  const int kb = t % (n / 16), rb = t / (n / 16);
  const int r = rb * 32 + j, i = kb * 16 + q * 8;
  *reinterpret_cast<u32x4 *>(dst + o * 8) = *reinterpret_cast<const u32x4 *>(src + (size_t)r * n + i);
}

// Output piece index o = ((kb*(m/32) + cb)*2 + q)*32 + j holds rows 16kb+8q+(0..7) of column 32cb+j.
__global__ void to_mfma16_u(const uint16_t *__restrict__ src, int R, int m, uint16_t *__restrict__ dst) {
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = (size_t)R * m / 8;
  if (o >= total) return;
  const int j = o & 31, q = (o >> 5) & 1;
  const size_t t = o >> 6;
  const int cb = t % (m / 32), kb = t / (m / 32);
  const int c = cb * 32 + j, r0 = kb * 16 + q * 8;
  uint16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = src[(size_t)(r0 + e) * m + c];
  u32x4 w;
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = (uint32_t)v[2 * e] | ((uint32_t)v[2 * e + 1] << 16);
  *reinterpret_cast<u32x4 *>(dst + o * 8) = w;
}

static int launch_pack(const parse_layer *L, const int32_t *subset, int subset_stride, int k, const int32_t *rep,
                       const int32_t *slot, const uint8_t *skip, int n_slots, const int32_t *n_patterns,
                       int max_patterns, void *Vt_S, void *Ut_S, hipStream_t s) {
  int st = check_layer(L);
  if (st != PARSE_OK) return st;
  if (!subset || !Vt_S || !Ut_S) return PARSE_EINVAL;
  if (k <= 0 || max_patterns <= 0 || n_slots <= 0) return PARSE_EINVAL;
  if (k > L->G || subset_stride < k || max_patterns > (1 << 24)) return PARSE_ESHAPE;
  if (!aligned16(Vt_S) || !aligned16(Ut_S)) return PARSE_EALIGN;
  const size_t gs = L->R / L->G, es = elem_size(L->dtype);
  const size_t vb = gs * L->n * es, ub = gs * L->m * es;  // multiples of 16 (checked by check_layer)
  const size_t big = vb > ub ? vb : ub;
  const long long tasks = (long long)((big + kCopyChunk - 1) / kCopyChunk) * 2 * k * max_patterns;
  const unsigned grid = (unsigned)(tasks < 1024 ? tasks : 1024);   // four workgroups per compute unit walk the list
  hipLaunchKernelGGL(pack_slabs, dim3(grid), dim3(kCopyThreads), 0, s, (const char *)L->Vt, (const char *)L->Ut, vb, ub,
                     L->G, k, subset, subset_stride, rep, slot, skip, n_slots, n_patterns, max_patterns, (char *)Vt_S,
                     (char *)Ut_S);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // namespace parse

using namespace parse;

extern "C" {

int parse_pack_experts(const parse_layer *L, const int32_t *subset, int32_t k, void *Vt_S, void *Ut_S,
                       parse_stream stream) {
  return launch_pack(L, subset, k, k, nullptr, nullptr, nullptr, 1, nullptr, 1, Vt_S, Ut_S, (hipStream_t)stream);
}

int parse_pack_patterns(const parse_layer *L, const int32_t *subset, int32_t subset_stride, int32_t k,
                        const int32_t *rep, const int32_t *n_patterns, int32_t max_patterns, void *Vt_S, void *Ut_S,
                        parse_stream stream) {
  return launch_pack(L, subset, subset_stride, k, rep, nullptr, nullptr, max_patterns, n_patterns, max_patterns, Vt_S,
                     Ut_S, (hipStream_t)stream);
}

int parse_pack_new_entries(const parse_layer *L, const int32_t *subset, int32_t subset_stride, int32_t k, int32_t P,
                           const int32_t *entry, const uint8_t *hit, int32_t n_slots, void *Vt_S, void *Ut_S,
                           parse_stream stream) {
  if (!entry || !hit) return PARSE_EINVAL;
  return launch_pack(L, subset, subset_stride, k, nullptr, entry, hit, n_slots, nullptr, P, Vt_S, Ut_S,
                     (hipStream_t)stream);
}

int parse_layer_to_mfma16(const parse_layer *src, void *Vt_out, void *Ut_out, parse_stream stream) {
  int st = check_layer(src);
  if (st != PARSE_OK) return st;
  if (!Vt_out || !Ut_out) return PARSE_EINVAL;
  if (src->dtype != PARSE_BF16 || src->layout != PARSE_ROWMAJOR) return PARSE_ELAYOUT;
  const int gs = src->R / src->G;
  if (src->n % 16 != 0 || src->m % 32 != 0 || gs % 32 != 0) return PARSE_ESHAPE;
  if (!aligned16(Vt_out) || !aligned16(Ut_out)) return PARSE_EALIGN;
  hipStream_t s = (hipStream_t)stream;
  const size_t nv = (size_t)src->R * src->n / 8, nu = (size_t)src->R * src->m / 8;
  hipLaunchKernelGGL(to_mfma16_v, dim3((unsigned)((nv + 255) / 256)), dim3(256), 0, s, (const uint16_t *)src->Vt,
                     src->R, src->n, (uint16_t *)Vt_out);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(to_mfma16_u, dim3((unsigned)((nu + 255) / 256)), dim3(256), 0, s, (const uint16_t *)src->Ut,
                     src->R, src->m, (uint16_t *)Ut_out);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // extern "C"
