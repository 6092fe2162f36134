// a7: decode step for bf16 PARSE_MFMA16 layers (Sec. 4.3, "Rank Reuse for Decoding"): every sequence keeps the
// rank subset chosen at prefill; one token per sequence.  Bandwidth-bound: the kernels stream each rank group
// that ANY sequence of the batch selected exactly once, straight from the layer's factor store in operand
// order (1 KiB coalesced per wavefront instruction, no LDS hop, no packed copies), and apply it to all
// sequences at once on the matrix cores (32 sequences = the N side of a 32x32x16 instruction).  A sequence
// whose pattern does not hold a group gets a zero in that group's part of z, so it contributes nothing.
//
//   decode_z     z partials: workgroup = (32-rank block, slice of the reduction axis n); its wavefronts split
//                the slice and reduce through LDS; skipped entirely if no sequence uses the block's group.
//   decode_zfin  adds the slices in order, masks by pattern membership, rounds to bf16 and lays z out in
//                operand order for phase 2 (tiny).
//   decode_y     workgroup = one 32-column block of the output; its wavefronts split the selected ranks,
//                reduce through LDS and store y as bf16.
// The streaming loops are branch-free: a wavefront's operand list is walked in chunks of DEC_CHUNK fetches, two
// chunks in flight (ping-pong registers), indices past the end are clamped to the last valid operand and their
// contribution is switched off by zeroing the small operand.
#include "common.hpp"

namespace parse {

constexpr int DZ_WAVES = 4, DZ_THREADS = DZ_WAVES * 64;
constexpr int DY_WAVES = 8, DY_THREADS = DY_WAVES * 64;
constexpr int DEC_CHUNK = 8;   // operand pairs fetched per chunk; two chunks in flight per wavefront
constexpr int DEC_MAXG = 64;

__device__ __forceinline__ bf16x8 dec_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// sequence b (< B <= 32) holds group g in its pattern
__device__ __forceinline__ bool seq_uses_group(const int32_t *__restrict__ subsets, int stride, int k, int n_patterns,
                                               const int32_t *__restrict__ pattern_id, int B, int b, int g) {
  if (b >= B) return false;
  const int pid = pattern_id[b];
  if (pid < 0 || pid >= n_patterns) return false;
  bool u = false;
  for (int i = 0; i < k; ++i) u = u || (subsets[(size_t)pid * stride + i] == g);
  return u;
}

// Per-group sequence masks built by the whole workgroup with two dependent loads per lane: lane t looks at entry
// i = t / 32 (+ blockDim/32 ...) of sequence b = t % 32's pattern and ORs bit b into gmask[that group].
// gmask (LDS, DEC_MAXG words) must be zeroed by the caller before; ends with a barrier.
__device__ __forceinline__ void build_group_masks(const int32_t *__restrict__ subsets, int stride, int k,
                                                  int n_patterns, const int32_t *__restrict__ pattern_id, int B, int G,
                                                  uint32_t *gmask) {
  const int b = threadIdx.x & 31;
  int pid = -1;
  if (b < B) pid = pattern_id[b];
  const bool ok = pid >= 0 && pid < n_patterns;
  for (int i = threadIdx.x >> 5; i < k; i += blockDim.x >> 5) {
    if (ok) {
      const int g = subsets[(size_t)pid * stride + i];
      if (g >= 0 && g < G) atomicOr(&gmask[g], 1u << b);
    }
  }
  __syncthreads();
}

// acc += sum over steps s in [0, cnt) of A_s x B_s, where A_s is the 1 KiB operand at a + s*a_step (elements,
// already lane-adjusted) and B_s the operand at b + idx(s)*b_step.  `bvalid` false zeroes this lane's B data.
template <typename IdxA, typename IdxB>
__device__ __forceinline__ void stream_mfma(const uint16_t *__restrict__ a, const uint16_t *__restrict__ b, int cnt,
                                            bool bvalid, IdxA a_off, IdxB b_off, f32x16 &acc) {
  if (cnt <= 0) return;
  u32x4 A0[DEC_CHUNK], B0[DEC_CHUNK], A1[DEC_CHUNK], B1[DEC_CHUNK];
  const u32x4 zero = {0, 0, 0, 0};
  auto load = [&](u32x4 *A, u32x4 *Bv, int base) {
#pragma unroll
    for (int i = 0; i < DEC_CHUNK; ++i) {
      const int s = min(base + i, cnt - 1);
      A[i] = *reinterpret_cast<const u32x4 *>(a + a_off(s));
      Bv[i] = *reinterpret_cast<const u32x4 *>(b + b_off(s));
    }
  };
  auto compute = [&](const u32x4 *A, const u32x4 *Bv, int base) {
#pragma unroll
    for (int i = 0; i < DEC_CHUNK; ++i) {
      const u32x4 bv = (bvalid && base + i < cnt) ? Bv[i] : zero;
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(A[i]), dec_bf16x8(bv), acc, 0, 0, 0);
    }
  };
  load(A0, B0, 0);
  for (int c0 = 0; c0 < cnt; c0 += 2 * DEC_CHUNK) {
    load(A1, B1, c0 + DEC_CHUNK);
    __builtin_amdgcn_sched_barrier(0);
    compute(A0, B0, c0);
    __builtin_amdgcn_sched_barrier(0);
    load(A0, B0, c0 + 2 * DEC_CHUNK);
    __builtin_amdgcn_sched_barrier(0);
    compute(A1, B1, c0 + DEC_CHUNK);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// grid (R/32, KS)
__global__ __launch_bounds__(DZ_THREADS) void decode_z(const uint16_t *__restrict__ Vt, const uint16_t *__restrict__ x,
                                                       int B, int n, int R, int gs, const int32_t *__restrict__ subsets,
                                                       int stride, int k, int n_patterns,
                                                       const int32_t *__restrict__ pattern_id, int KS,
                                                       float *__restrict__ zp) {
  __shared__ float red[DZ_WAVES - 1][16][64];
  __shared__ uint32_t gmask[DEC_MAXG];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, q = lane >> 5;
  const int rb = blockIdx.x, ks = blockIdx.y;
  const int g = rb * 32 / gs;
  if (threadIdx.x < DEC_MAXG) gmask[threadIdx.x] = 0;
  __syncthreads();
  build_group_masks(subsets, stride, k, n_patterns, pattern_id, B, R / gs, gmask);
  if (gmask[g] == 0u) return;   // nobody selected this group: nothing is read
  const int nkb = n / 16;
  const int w0 = (int)(((long long)nkb * ks) / KS), w1 = (int)(((long long)nkb * (ks + 1)) / KS);
  const int len = w1 - w0;
  const int s0 = w0 + (len * wave) / DZ_WAVES, s1 = w0 + (len * (wave + 1)) / DZ_WAVES;
  const uint16_t *vbase = Vt + (((size_t)rb * nkb + s0) * 64 + lane) * 8;
  const uint16_t *xrow = x + (size_t)min(l32, B - 1) * n + (size_t)s0 * 16 + q * 8;
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  stream_mfma(vbase, xrow, s1 - s0, l32 < B, [](int s) { return (size_t)s * 512; },
              [](int s) { return (size_t)s * 16; }, acc);
  if (wave > 0) {
#pragma unroll
    for (int e = 0; e < 16; ++e) red[wave - 1][e][lane] = acc[e];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int w = 0; w < DZ_WAVES - 1; ++w)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] += red[w][e][lane];
    // lane: sequence l32, ranks rb*32 + 8*blk + 4*q + (0..3)
    float *dst = zp + ((size_t)ks * 32 + l32) * R + rb * 32 + q * 4;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
      *reinterpret_cast<float4 *>(dst + blk * 8) = float4{acc[blk * 4], acc[blk * 4 + 1], acc[blk * 4 + 2], acc[blk * 4 + 3]};
  }
}

// one thread per 16-byte operand piece of z: piece o = (kb*2 + q)*32 + b holds z[b][16kb + 8q + (0..7)]
__global__ void decode_zfin(const float *__restrict__ zp, int KS, int B, int R, int gs,
                            const int32_t *__restrict__ subsets, int stride, int k, int n_patterns,
                            const int32_t *__restrict__ pattern_id, uint16_t *__restrict__ zf,
                            int32_t *__restrict__ used_out /* [0] = count, [1..] = group ids ascending */) {
  __shared__ uint32_t gmask[DEC_MAXG];
  const int G = R / gs;
  if (threadIdx.x < DEC_MAXG) gmask[threadIdx.x] = 0;
  __syncthreads();
  build_group_masks(subsets, stride, k, n_patterns, pattern_id, B, G, gmask);
  if (blockIdx.x == 0 && threadIdx.x < 64) {   // the groups selected by at least one sequence, for phase 2
    const int lane = threadIdx.x;
    const bool u = lane < G && gmask[lane] != 0u;
    const unsigned long long mask = __ballot(u);
    if (u) used_out[1 + __popcll(mask & ((1ull << lane) - 1ull))] = lane;
    if (lane == 0) used_out[0] = __popcll(mask);
  }
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= R * 4) return;   // R/16 * 64 pieces
  const int b = o & 31, q = (o >> 5) & 1, kb = o >> 6;
  const int r0 = kb * 16 + q * 8;
  const int g = r0 / gs;
  float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if ((gmask[g] >> b) & 1u) {
    for (int s = 0; s < KS; ++s) {
      const float *src = zp + ((size_t)s * 32 + b) * R + r0;
      const float4 a = *reinterpret_cast<const float4 *>(src), c = *reinterpret_cast<const float4 *>(src + 4);
      v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
      v[4] += c.x; v[5] += c.y; v[6] += c.z; v[7] += c.w;
    }
  }
  u32x4 w;
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(v[2 * e], v[2 * e + 1]);
  *reinterpret_cast<u32x4 *>(zf + (size_t)o * 8) = w;
}

// grid (m/32)
__global__ __launch_bounds__(DY_THREADS) void decode_y(const uint16_t *__restrict__ Ut, const uint16_t *__restrict__ zf,
                                                       int B, int m, int R, int G, int gs,
                                                       const int32_t *__restrict__ used_in,
                                                       uint16_t *__restrict__ y) {
  __shared__ float red[DY_WAVES][16][64];
  __shared__ int32_t used[DEC_MAXG];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, q = lane >> 5;
  const int cb = blockIdx.x, ncb = m / 32;
  const int n_used = min(used_in[0], G);
  if (threadIdx.x < n_used) used[threadIdx.x] = used_in[1 + threadIdx.x];
  __syncthreads();
  const int kpg = gs / 16;                 // reduction blocks per group
  const int total = n_used * kpg;          // selected reduction blocks
  const int s0 = (total * wave) / DY_WAVES, s1 = (total * (wave + 1)) / DY_WAVES;
  const uint16_t *ubase = Ut + ((size_t)cb * 64 + lane) * 8;
  const uint16_t *zbase = zf + (size_t)lane * 8;
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  const size_t ustep = (size_t)ncb * 512;
  auto kb_of = [&](int s) { const int t = s0 + s; return used[t / kpg] * kpg + t % kpg; };
  stream_mfma(ubase, zbase, s1 - s0, true, [&](int s) { return (size_t)kb_of(s) * ustep; },
              [&](int s) { return (size_t)kb_of(s) * 512; }, acc);
#pragma unroll
  for (int e = 0; e < 16; ++e) red[wave][e][lane] = acc[e];
  __syncthreads();
  // 16 x 64 sums over the wavefronts
  for (int i = threadIdx.x; i < 16 * 64; i += DY_THREADS) {
    const int e = i >> 6, ln = i & 63;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < DY_WAVES; ++w) s += red[w][e][ln];
    red[0][e][ln] = s;   // each (e, ln) is read and written by this thread only
  }
  __syncthreads();
  // store: lane (of wave 0's layout) holds sequence l32, columns cb*32 + 8*blk + 4*q + (0..3)
  if (wave == 0 && l32 < B) {
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      u32x2 w;
      w[0] = pack_bf16x2(red[0][blk * 4 + 0][lane], red[0][blk * 4 + 1][lane]);
      w[1] = pack_bf16x2(red[0][blk * 4 + 2][lane], red[0][blk * 4 + 3][lane]);
      *reinterpret_cast<u32x2 *>(y + (size_t)l32 * m + cb * 32 + blk * 8 + q * 4) = w;
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// One-launch form.  Workgroups [0, w_lo) are phase-1 workers: each takes whole 32-rank blocks (all of n, its
// 8 wavefronts split the reduction axis and reduce through LDS), masks, rounds and stores z in operand order,
// then publishes the block with a release + counter increment and never waits.  Workgroups [w_lo, grid) are
// phase-2 workers: each owns a range of 32-column output blocks, fetches ALL its Ut operands into registers
// right away (they do not depend on z, so this traffic overlaps phase 1), then waits until the counter shows
// every rank block published, reads z (cache-resident) and finishes.  Phase-1 workers have the lower ids, so
// they are dispatched first and the wait always ends; the spin is bounded anyway and a timeout raises a flag.
// The two counters of a call live in a slot of a file-scope device array, start at zero and are put back to
// zero by the last phase-2 worker, so nothing has to be cleared between calls.
constexpr int DF_WAVES = 8, DF_THREADS = DF_WAVES * 64;
constexpr int DF_MAXU = 32;      // Ut operands a wavefront keeps in registers across the wait
constexpr int DF_SLOTS = 64;
constexpr unsigned DF_SPIN_LIMIT = 1u << 22;
__device__ unsigned g_dec_sync[DF_SLOTS][4];   // [slot]: 0 = rank blocks published, 1 = phase-2 workers past the wait, 2 = timeout flag

struct DfArgs {
  const uint16_t *Vt, *Ut, *x;
  uint16_t *y, *zf;
  const int32_t *subsets, *pattern_id;
  int stride, k, n_patterns, B, n, m, R, G, gs;
  int n1, w_lo, slot;
};

__global__ __launch_bounds__(DF_THREADS) void decode_fused(DfArgs a) {
  __shared__ float red[DF_WAVES][16][64];      // 32 KiB
  __shared__ uint32_t gmask[DEC_MAXG];
  __shared__ int32_t used[DEC_MAXG];
  __shared__ int32_t n_used_s;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, q = lane >> 5;
  const int wg = blockIdx.x;
  unsigned *sync = g_dec_sync[a.slot];
  if (threadIdx.x < DEC_MAXG) gmask[threadIdx.x] = 0;
  __syncthreads();
  build_group_masks(a.subsets, a.stride, a.k, a.n_patterns, a.pattern_id, a.B, a.G, gmask);

  if (wg < a.w_lo) {
    // ---------------------------------------------------------------- phase 1: z for whole rank blocks
    const int nkb = a.n / 16;
    for (int rb = wg; rb < a.n1; rb += a.w_lo) {
      const int g = rb * 32 / a.gs;
      const uint32_t gm = gmask[g];
      if (gm != 0u) {   // uniform over the workgroup
        const int s0 = (nkb * wave) / DF_WAVES, s1 = (nkb * (wave + 1)) / DF_WAVES;
        const uint16_t *vbase = a.Vt + (((size_t)rb * nkb + s0) * 64 + lane) * 8;
        const uint16_t *xrow = a.x + (size_t)min(l32, a.B - 1) * a.n + (size_t)s0 * 16 + q * 8;
        f32x16 acc;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = 0.f;
        stream_mfma(vbase, xrow, s1 - s0, l32 < a.B, [](int s) { return (size_t)s * 512; },
                    [](int s) { return (size_t)s * 16; }, acc);
#pragma unroll
        for (int e = 0; e < 16; ++e) red[wave][e][lane] = acc[e];
        __syncthreads();
        for (int i = threadIdx.x; i < 16 * 64; i += DF_THREADS) {
          const int e = i >> 6, ln = i & 63;
          float sum = 0.f;
#pragma unroll
          for (int w = 0; w < DF_WAVES; ++w) sum += red[w][e][ln];
          red[0][e][ln] = sum;
        }
        __syncthreads();
        // 128 lanes emit the block's z in operand order: piece (kbl, q2, b) = ranks 16 kbl + 8 q2 + (0..7) of sequence b
        if (threadIdx.x < 128) {
          const int b = threadIdx.x & 31, q2 = (threadIdx.x >> 5) & 1, kbl = threadIdx.x >> 6;
          const bool on = (gm >> b) & 1u;
          float v[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int r = 16 * kbl + 8 * q2 + j;       // rank inside the block
            const int e = 4 * (r / 8) + (r % 4), ln = 32 * ((r % 8) / 4) + b;
            v[j] = on ? red[0][e][ln] : 0.f;
          }
          u32x4 w;
#pragma unroll
          for (int j = 0; j < 4; ++j) w[j] = pack_bf16x2(v[2 * j], v[2 * j + 1]);
          *reinterpret_cast<u32x4 *>(a.zf + ((size_t)((rb * 2 + kbl) * 2 + q2) * 32 + b) * 8) = w;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // every lane's z stores are visible device-wide ...
        __syncthreads();                                     // ... before lane 0 publishes the block
      }
      if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        atomicAdd(&sync[0], 1u);
      }
    }
    return;
  }

  // ------------------------------------------------------------------ phase 2: y for a range of column blocks
  if (wave == 0) {
    const bool u = lane < a.G && gmask[lane] != 0u;
    const unsigned long long mask = __ballot(u);
    if (u) used[__popcll(mask & ((1ull << lane) - 1ull))] = lane;
    if (lane == 0) n_used_s = __popcll(mask);
  }
  __syncthreads();
  const int ncb = a.m / 32, kpg = a.gs / 16;
  const int total_kb = n_used_s * kpg;
  const int nw2 = gridDim.x - a.w_lo, j2 = wg - a.w_lo;
  const int c0 = (int)(((long long)ncb * j2) / nw2), c1 = (int)(((long long)ncb * (j2 + 1)) / nw2);
  const int units = (c1 - c0) * total_kb;
  const int u0 = (units * wave) / DF_WAVES, u1 = (units * (wave + 1)) / DF_WAVES;
  const int cnt = u1 - u0;
  const int cbl_first = total_kb > 0 ? u0 / total_kb : 0;   // local column block of this wave's first unit
  auto unit_kb = [&](int u) { const int kbi = u % total_kb; return used[kbi / kpg] * kpg + kbi % kpg; };
  auto unit_addr = [&](int u) {
    return a.Ut + (((size_t)unit_kb(u) * ncb + c0 + u / total_kb) * 64 + lane) * 8;
  };
  u32x4 ur[DF_MAXU];
  if (cnt > 0) {
#pragma unroll
    for (int i = 0; i < DF_MAXU; ++i) ur[i] = *reinterpret_cast<const u32x4 *>(unit_addr(min(u0 + i, u1 - 1)));
  }
  // wait for phase 1
  if (threadIdx.x == 0) {
    unsigned it = 0;
    while (__hip_atomic_load(&sync[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)a.n1) {
      if (++it > DF_SPIN_LIMIT) { atomicExch(&sync[2], 1u); break; }
      __builtin_amdgcn_s_sleep(4);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    const unsigned passed = atomicAdd(&sync[1], 1u) + 1u;
    if (passed == (unsigned)nw2) {   // every phase-2 worker is past the wait: hand the slot back clean
      atomicExch(&sync[0], 0u);
      atomicExch(&sync[1], 0u);
    }
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");

  f32x16 acc0, acc1;
#pragma unroll
  for (int e = 0; e < 16; ++e) { acc0[e] = 0.f; acc1[e] = 0.f; }
  const u32x4 zero = {0, 0, 0, 0};
  if (cnt > 0) {
    // the operands held in registers
#pragma unroll
    for (int c = 0; c < DF_MAXU; c += DEC_CHUNK) {
      u32x4 zr[DEC_CHUNK];
#pragma unroll
      for (int i = 0; i < DEC_CHUNK; ++i)
        zr[i] = *reinterpret_cast<const u32x4 *>(a.zf + ((size_t)unit_kb(min(u0 + c + i, u1 - 1)) * 64 + lane) * 8);
#pragma unroll
      for (int i = 0; i < DEC_CHUNK; ++i) {
        const int u = u0 + c + i;
        const bool live = u < u1;
        const bool second = live && (u / total_kb != cbl_first);
        const u32x4 z0 = (live && !second) ? zr[i] : zero, z1 = second ? zr[i] : zero;
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(ur[c + i]), dec_bf16x8(z0), acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(ur[c + i]), dec_bf16x8(z1), acc1, 0, 0, 0);
      }
    }
    // anything beyond the register budget is streamed now
    for (int c = DF_MAXU; c < cnt; c += DEC_CHUNK) {
      u32x4 uu[DEC_CHUNK], zr[DEC_CHUNK];
#pragma unroll
      for (int i = 0; i < DEC_CHUNK; ++i) {
        const int u = min(u0 + c + i, u1 - 1);
        uu[i] = *reinterpret_cast<const u32x4 *>(unit_addr(u));
        zr[i] = *reinterpret_cast<const u32x4 *>(a.zf + ((size_t)unit_kb(u) * 64 + lane) * 8);
      }
#pragma unroll
      for (int i = 0; i < DEC_CHUNK; ++i) {
        const int u = u0 + c + i;
        const bool live = u < u1;
        const bool second = live && (u / total_kb != cbl_first);
        const u32x4 z0 = (live && !second) ? zr[i] : zero, z1 = second ? zr[i] : zero;
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(uu[i]), dec_bf16x8(z0), acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(uu[i]), dec_bf16x8(z1), acc1, 0, 0, 0);
      }
    }
  }
  // per local column block: add the wavefronts' contributions in wave order and store
  for (int jl = 0; jl < c1 - c0; ++jl) {
    const bool first = cnt > 0 && cbl_first == jl, second = cnt > 0 && cbl_first + 1 == jl;
#pragma unroll
    for (int e = 0; e < 16; ++e) red[wave][e][lane] = first ? acc0[e] : (second ? acc1[e] : 0.f);
    __syncthreads();
    for (int i = threadIdx.x; i < 16 * 64; i += DF_THREADS) {
      const int e = i >> 6, ln = i & 63;
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < DF_WAVES; ++w) sum += red[w][e][ln];
      red[0][e][ln] = sum;
    }
    __syncthreads();
    if (wave == 0 && l32 < a.B) {
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        u32x2 w;
        w[0] = pack_bf16x2(red[0][blk * 4 + 0][lane], red[0][blk * 4 + 1][lane]);
        w[1] = pack_bf16x2(red[0][blk * 4 + 2][lane], red[0][blk * 4 + 3][lane]);
        *reinterpret_cast<u32x2 *>(a.y + (size_t)l32 * a.m + (c0 + jl) * 32 + blk * 8 + q * 4) = w;
      }
    }
    __syncthreads();
  }
}

static int g_decode_schedule = 0;   // 0 = one launch when the shape allows, 1 = always three launches
void set_decode_schedule(int v) { g_decode_schedule = v; }

static int decode_slices(int R) {
  int ks = (640 + R / 32 - 1) / (R / 32);
  if (ks < 1) ks = 1;
  if (ks > 16) ks = 16;
  return ks;
}

size_t decode_workspace_bytes(const parse_layer *L) {
  const int KS = decode_slices(L->R);
  return round_up((size_t)KS * 32 * L->R * sizeof(float), 256) + round_up((size_t)L->R * 32 * sizeof(uint16_t), 256) +
         round_up((DEC_MAXG + 1) * sizeof(int32_t), 256);
}

int forward_decode_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *x, int B,
                        const int32_t *pattern_id, uint16_t *y, void *workspace, hipStream_t s) {
  const int gs = L->R / L->G;
  const int KS = decode_slices(L->R);
  static int n_cu = 0;
  static unsigned call_index = 0;
  if (n_cu == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    PARSE_HIP_TRY(hipGetDevice(&dev));
    PARSE_HIP_TRY(hipGetDeviceProperties(&prop, dev));
    n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  const int n1 = L->R / 32, ncb = L->m / 32;
  // one launch: phase-1 workers are a minority of the grid, every phase-2 wavefront sees at most two column blocks
  const int w_lo = n1 < n_cu / 2 ? n1 : 0;
  if (g_decode_schedule == 0 && w_lo > 0 && (ncb + (n_cu - w_lo) - 1) / (n_cu - w_lo) <= DF_WAVES && L->n / 16 >= DF_WAVES) {
    uint16_t *zf1 = reinterpret_cast<uint16_t *>((char *)workspace + round_up((size_t)KS * 32 * L->R * sizeof(float), 256));
    DfArgs a{(const uint16_t *)L->Vt, (const uint16_t *)L->Ut, x, y, zf1, pt->subsets, pattern_id, pt->subset_stride,
             pt->k, pt->n_patterns, B, L->n, L->m, L->R, L->G, gs, n1, w_lo, (int)(call_index++ % DF_SLOTS)};
    hipLaunchKernelGGL(decode_fused, dim3(n_cu), dim3(DF_THREADS), 0, s, a);
    PARSE_LAUNCH_CHECK();
    return PARSE_OK;
  }
  float *zp = reinterpret_cast<float *>(workspace);
  uint16_t *zf = reinterpret_cast<uint16_t *>((char *)workspace + round_up((size_t)KS * 32 * L->R * sizeof(float), 256));
  int32_t *used = reinterpret_cast<int32_t *>((char *)zf + round_up((size_t)L->R * 32 * sizeof(uint16_t), 256));
  hipLaunchKernelGGL(decode_z, dim3(L->R / 32, KS), dim3(DZ_THREADS), 0, s, (const uint16_t *)L->Vt, x, B, L->n, L->R,
                     gs, pt->subsets, pt->subset_stride, pt->k, pt->n_patterns, pattern_id, KS, zp);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(decode_zfin, dim3((L->R * 4 + 255) / 256), dim3(256), 0, s, zp, KS, B, L->R, gs, pt->subsets,
                     pt->subset_stride, pt->k, pt->n_patterns, pattern_id, zf, used);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(decode_y, dim3(L->m / 32), dim3(DY_THREADS), 0, s, (const uint16_t *)L->Ut, zf, B, L->m, L->R,
                     L->G, gs, used, y);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // namespace parse
