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
// One-launch form: a persistent grid of one workgroup per compute unit (a compute unit sustains roughly 50 GB/s
// of cache-line fills, so HBM rate needs every unit streaming in every phase).
//   A  z partials.  Task = (four consecutive 32-rank blocks, slice s of the S slices of n); a workgroup takes
//      task ids wg, wg + grid, ...  The slice of the token rows x is staged in LDS once (coalesced row reads)
//      and shared by the four rank blocks; wavefront w owns rank block w % 4 and half w / 4 of the slice, its
//      Vt operands come straight from the store; the two halves add up through LDS; fp32 partials go to the
//      workspace.  Rank blocks of groups nobody selected are skipped.
//   B  every wavefront requests the Ut operands of its share of phase D right away (registers plus an LDS stash):
//      they do not depend on z, so this stream overlaps the two grid barriers and phase C.
//   -- grid barrier --
//   C  z: each workgroup adds the S partials of its share of z in slice order, masks by pattern membership,
//      rounds to bf16 and stores z in operand order.
//   -- grid barrier --
//   D  y: a workgroup owns up to two 32-column output blocks; wavefront w owns an eighth of the selected
//      reduction blocks, reads their z operands (cache-resident), multiplies with the operands it already
//      holds, and the eight wavefronts add up through LDS.
// The grid barriers count arrivals in a slot of a file-scope device array; the last arriver raises DF_FLAGS
// "go" words in separate cache lines so the waiters do not all poll one address.  Waits are bounded (a timeout
// raises a sticky flag and lets the kernel run to its end).  The last workgroup past the second barrier puts
// the slot back to zero, so nothing has to be cleared between calls.  The launch is cooperative: all
// workgroups are resident together.
constexpr int DF_WAVES = 8, DF_THREADS = DF_WAVES * 64;
constexpr int DF_MAXK = 16;      // selected reduction blocks whose Ut operands a wavefront keeps in registers across the barriers
constexpr int DF_STASH = 6;      // further reduction blocks per wavefront whose Ut operands wait in LDS
constexpr int DF_SLOTS = 64;
constexpr int DF_FLAGS = 32;
constexpr int DF_MAXSLICE = 64;  // reduction steps (of 16 columns) of x staged per task
constexpr int DF_XLD = DF_MAXSLICE * 16 + 8;
constexpr int DF_MAXKB = 1024;   // selected reduction blocks a worker can list
constexpr unsigned DF_SPIN_LIMIT = 1u << 20;
struct DfBarrier {
  unsigned arrived;
  unsigned pad[15];
  unsigned go[DF_FLAGS][16];     // one word per 64-byte line
};
struct DfSync {
  DfBarrier bar[2];
  unsigned passed;               // workgroups past the second barrier
  unsigned timeout;              // sticky: a wait gave up
  unsigned pad[14];
};
__device__ DfSync g_dec_sync[DF_SLOTS];

struct DfArgs {
  const uint16_t *Vt, *Ut, *x;
  uint16_t *y, *zf;
  float *zp;
  const int32_t *subsets, *pattern_id;
  int stride, k, n_patterns, B, n, m, R, G, gs;
  int S, slot;
  long long *stamps;   // diagnostics build only: 8 timestamps per workgroup
};

#ifdef PARSE_DEC_TIMING
#define DEC_STAMP(i) do { if (threadIdx.x == 0) a.stamps[(size_t)blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#else
#define DEC_STAMP(i) do {} while (0)
#endif

// All workgroups of the grid arrive; lane 0 of each spins (bounded) on one of the go words.  Ends with a
// workgroup barrier; writes made before it by any workgroup are visible after it.
__device__ __forceinline__ void grid_barrier(DfBarrier *bar, unsigned *timeout_flag) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    const unsigned n = atomicAdd(&bar->arrived, 1u) + 1u;
    if (n == gridDim.x) {
      for (int f = 0; f < DF_FLAGS; ++f) __hip_atomic_store(&bar->go[f][0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      unsigned it = 0;
      unsigned *flag = &bar->go[blockIdx.x % DF_FLAGS][0];
      while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
        if (++it > DF_SPIN_LIMIT) { atomicExch(timeout_flag, 1u); break; }
        __builtin_amdgcn_s_sleep(8);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
  __syncthreads();
}

__global__ __launch_bounds__(DF_THREADS) void decode_persist(DfArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char df_lds[];
  float (*red)[16][64] = reinterpret_cast<float (*)[16][64]>(df_lds);                        // [DF_WAVES] 32 KiB
  uint16_t *xs = reinterpret_cast<uint16_t *>(df_lds + DF_WAVES * 16 * 64 * sizeof(float));   // phase A: [32][DF_XLD]
  int32_t *kb_list = reinterpret_cast<int32_t *>(xs);                                         // phases B-D: [DF_MAXKB]
  uint16_t *stash = xs + DF_MAXKB * 2;                                                        // [DF_WAVES][DF_STASH][2][512]
  __shared__ uint32_t gmask[DEC_MAXG];
  __shared__ int32_t used[DEC_MAXG];
  __shared__ int32_t n_used_s;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, q = lane >> 5;
  const int wg = blockIdx.x, nwg = gridDim.x;
  DfSync *sync = &g_dec_sync[a.slot];
  DEC_STAMP(0);
  if (threadIdx.x < DEC_MAXG) gmask[threadIdx.x] = 0;
  __syncthreads();
  build_group_masks(a.subsets, a.stride, a.k, a.n_patterns, a.pattern_id, a.B, a.G, gmask);

  // ------------------------------------------------------------------ A: z partials
  {
    const int nkb = a.n / 16, nrb = a.R / 32, nquads = (nrb + 3) / 4;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const int rbl = wave_s & 3, half = wave_s >> 2;
    for (int task = wg; task < nquads * a.S; task += nwg) {
      const int quad = task / a.S, sl = task - quad * a.S;
      const int w0 = (int)(((long long)nkb * sl) / a.S), w1 = (int)(((long long)nkb * (sl + 1)) / a.S);
      const int len = w1 - w0;                               // <= DF_MAXSLICE (host)
      // any of the quad's rank blocks selected?
      bool any = false;
      for (int i = 0; i < 4; ++i) {
        const int r = quad * 4 + i;
        any = any || (r < nrb && gmask[r * 32 / a.gs] != 0u);
      }
      if (!any) continue;   // uniform
      __syncthreads();      // earlier readers of xs / red are done
      // stage x[:, 16 w0 .. 16 w1): rows of len*32 bytes in 16-byte pieces, zero rows beyond B.  All of a lane's
      // pieces (at most 8) are requested before the first one is stored.
      const int ppr = len * 2;                               // pieces per row
      u32x4 xp[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int piece = min(i * DF_THREADS + (int)threadIdx.x, 32 * ppr - 1);
        const int r = piece / ppr, c = (piece - r * ppr) * 8;
        xp[i] = *reinterpret_cast<const u32x4 *>(a.x + (size_t)min(r, a.B - 1) * a.n + (size_t)w0 * 16 + c);
      }
      const int rb = quad * 4 + rbl;
      const bool live = rb < nrb && gmask[min(rb, nrb - 1) * 32 / a.gs] != 0u;   // uniform per wavefront
      const int h0 = (len * half) / 2, h1 = (len * (half + 1)) / 2;             // this wavefront's steps of the slice
      const int cnt = live ? h1 - h0 : 0;
      f32x16 acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
      const char *vblock = reinterpret_cast<const char *>(a.Vt) + ((size_t)min(rb, nrb - 1) * nkb + w0 + h0) * 1024;
      const uint32_t lane_off = lane * 16;
      // Vt operands: chunks of DEC_CHUNK, two chunks in flight; the first two are requested before the x slice is ready
      u32x4 V0[DEC_CHUNK], V1[DEC_CHUNK];
      auto load_v = [&](u32x4 *V, int base) {
#pragma unroll
        for (int i = 0; i < DEC_CHUNK; ++i)
          V[i] = *reinterpret_cast<const u32x4 *>(vblock + (size_t)max(min(base + i, cnt - 1), 0) * 1024 + lane_off);
      };
      load_v(V0, 0);
      load_v(V1, DEC_CHUNK);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int piece = i * DF_THREADS + threadIdx.x;
        if (piece < 32 * ppr) {
          const int r = piece / ppr, c = (piece - r * ppr) * 8;
          *reinterpret_cast<u32x4 *>(xs + r * DF_XLD + c) = r < a.B ? xp[i] : u32x4{0, 0, 0, 0};
        }
      }
      __syncthreads();      // x slice staged
      const uint16_t *xb_base = xs + l32 * DF_XLD + h0 * 16 + q * 8;
      const u32x4 zero = {0, 0, 0, 0};
      auto compute = [&](const u32x4 *V, int base) {
#pragma unroll
        for (int i = 0; i < DEC_CHUNK; ++i) {
          const int st = min(base + i, max(cnt - 1, 0));
          const u32x4 xv = *reinterpret_cast<const u32x4 *>(xb_base + st * 16);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(V[i]), dec_bf16x8(base + i < cnt ? xv : zero), acc, 0, 0, 0);
        }
      };
      for (int c0 = 0; c0 < cnt; c0 += 2 * DEC_CHUNK) {
        compute(V0, c0);
        __builtin_amdgcn_sched_barrier(0);
        load_v(V0, c0 + 2 * DEC_CHUNK);
        __builtin_amdgcn_sched_barrier(0);
        compute(V1, c0 + DEC_CHUNK);
        __builtin_amdgcn_sched_barrier(0);
        load_v(V1, c0 + 3 * DEC_CHUNK);
        __builtin_amdgcn_sched_barrier(0);
      }
      // halves add up: wavefronts 4..7 hand their tile to 0..3
      if (half == 1) {
#pragma unroll
        for (int e = 0; e < 16; ++e) red[rbl][e][lane] = acc[e];
      }
      __syncthreads();
      if (half == 0 && live) {
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] += red[rbl][e][lane];
        // lane: sequence l32, ranks rb*32 + 8*blk + 4*q + (0..3)
        float *dst = a.zp + ((size_t)sl * 32 + l32) * a.R + rb * 32 + q * 4;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
          *reinterpret_cast<float4 *>(dst + blk * 8) = float4{acc[blk * 4], acc[blk * 4 + 1], acc[blk * 4 + 2], acc[blk * 4 + 3]};
      }
    }
  }
  DEC_STAMP(1);
  __syncthreads();   // xs is about to be reused as the kb list

  // ------------------------------------------------------------------ B: request the Ut operands of phase D
  if (wave == 0) {
    const bool u = lane < a.G && gmask[lane] != 0u;
    const unsigned long long mask = __ballot(u);
    if (u) used[__popcll(mask & ((1ull << lane) - 1ull))] = lane;
    if (lane == 0) n_used_s = __popcll(mask);
  }
  __syncthreads();
  const int ncb = a.m / 32, kpg = a.gs / 16;
  const int total_kb = n_used_s * kpg;
  for (int i = threadIdx.x; i < total_kb; i += DF_THREADS) kb_list[i] = used[i / kpg] * kpg + i % kpg;
  __syncthreads();
  const int c0 = (int)(((long long)ncb * wg) / nwg), c1 = (int)(((long long)ncb * (wg + 1)) / nwg);
  const int nc = c1 - c0;                                    // 0, 1 or 2 column blocks (checked on the host)
  // wave w owns selected reduction blocks [k0, k1) for all of the worker's column blocks: one z operand feeds nc products
  const int k0 = (total_kb * wave) / DF_WAVES, k1 = (total_kb * (wave + 1)) / DF_WAVES;
  const int cnt = nc > 0 ? k1 - k0 : 0;
  const uint16_t *ubase = a.Ut + ((size_t)c0 * 64 + lane) * 8;
  const size_t ustep = (size_t)ncb * 512;
  const int second_off = nc > 1 ? 512 : 0;
  u32x4 ur[DF_MAXK][2];
  if (cnt > 0) {
#pragma unroll
    for (int i = 0; i < DF_MAXK; ++i) {
      const uint16_t *src = ubase + (size_t)kb_list[k0 + min(i, cnt - 1)] * ustep;
      ur[i][0] = *reinterpret_cast<const u32x4 *>(src);
      if (nc > 1) ur[i][1] = *reinterpret_cast<const u32x4 *>(src + 512);   // uniform over the workgroup
    }
  }
  // operands past the register budget wait in this wavefront's LDS stash (lane-linear, conflict-free)
  uint16_t *my_stash = stash + (size_t)wave * DF_STASH * 2 * 512 + lane * 8;
  const int nstash = min(max(cnt - DF_MAXK, 0), DF_STASH);
  if (nstash > 0) {
#pragma unroll
    for (int h = 0; h < DF_STASH; h += 3) {   // three reduction blocks at a time keep the staging registers few
      u32x4 tmp[3][2];
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        const uint16_t *src = ubase + (size_t)kb_list[k0 + min(DF_MAXK + h + i, cnt - 1)] * ustep;
        tmp[i][0] = *reinterpret_cast<const u32x4 *>(src);
        tmp[i][1] = *reinterpret_cast<const u32x4 *>(src + second_off);
      }
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        *reinterpret_cast<u32x4 *>(my_stash + ((h + i) * 2 + 0) * 512) = tmp[i][0];
        *reinterpret_cast<u32x4 *>(my_stash + ((h + i) * 2 + 1) * 512) = tmp[i][1];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  DEC_STAMP(2);
  grid_barrier(&sync->bar[0], &sync->timeout);
  DEC_STAMP(3);

  // ------------------------------------------------------------------ C: z = sum of the slices, masked, bf16, operand order
  {
    // This workgroup's pieces of z (16-byte pieces: o = (kb*2 + q)*32 + b).  Lane (slice, piece) fetches one
    // 32-byte partial, so all S slices of a piece are in flight together; the sums are then taken in slice order.
    const int pieces = a.R * 4;
    const int o_lo = (int)(((long long)pieces * wg) / nwg), o_hi = (int)(((long long)pieces * (wg + 1)) / nwg);
    float *part = reinterpret_cast<float *>(red);            // [DF_THREADS][8] staging, 16 KiB of the 32 KiB
    const int per_round = DF_THREADS / a.S;                  // pieces handled per round (S <= DF_MAX_SLICES <= 64)
    for (int base = o_lo; base < o_hi; base += per_round) {
      const int pl = threadIdx.x / a.S, sl = threadIdx.x - pl * a.S;   // piece within the round, slice
      const int o = base + pl;
      const bool mine = pl < per_round && o < o_hi;
      float4 f0 = {0, 0, 0, 0}, f1 = {0, 0, 0, 0};
      if (mine) {
        const int b = o & 31, q2 = (o >> 5) & 1, kb = o >> 6;
        const int r0 = kb * 16 + q2 * 8;
        if ((gmask[r0 / a.gs] >> b) & 1u) {
          const float *src = a.zp + ((size_t)sl * 32 + b) * a.R + r0;
          f0 = *reinterpret_cast<const float4 *>(src);
          f1 = *reinterpret_cast<const float4 *>(src + 4);
        }
      }
      __syncthreads();
      *reinterpret_cast<float4 *>(part + (size_t)threadIdx.x * 8) = f0;
      *reinterpret_cast<float4 *>(part + (size_t)threadIdx.x * 8 + 4) = f1;
      __syncthreads();
      if (threadIdx.x < per_round && base + (int)threadIdx.x < o_hi) {
        float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int s2 = 0; s2 < a.S; ++s2) {
          const float *pp = part + ((size_t)threadIdx.x * a.S + s2) * 8;
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += pp[e];
        }
        u32x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(v[2 * e], v[2 * e + 1]);
        *reinterpret_cast<u32x4 *>(a.zf + (size_t)(base + threadIdx.x) * 8) = w;
      }
    }
  }
  DEC_STAMP(7);
  grid_barrier(&sync->bar[1], &sync->timeout);
  if (threadIdx.x == 0) {
    const unsigned passed = atomicAdd(&sync->passed, 1u) + 1u;
    if (passed == (unsigned)nwg) {   // everybody is past both barriers: hand the slot back clean
      for (int bi = 0; bi < 2; ++bi) {
        for (int f = 0; f < DF_FLAGS; ++f)
          __hip_atomic_store(&sync->bar[bi].go[f][0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        atomicExch(&sync->bar[bi].arrived, 0u);
      }
      atomicExch(&sync->passed, 0u);
    }
  }
  DEC_STAMP(4);

  // ------------------------------------------------------------------ D: y
  f32x16 acc0, acc1;
#pragma unroll
  for (int e = 0; e < 16; ++e) { acc0[e] = 0.f; acc1[e] = 0.f; }
  const u32x4 zero = {0, 0, 0, 0};
  const uint16_t *zbase = a.zf + (size_t)lane * 8;
  if (cnt > 0) {
    // all z operands of the register-held part are requested at once
    u32x4 zr[DF_MAXK];
#pragma unroll
    for (int i = 0; i < DF_MAXK; ++i) zr[i] = *reinterpret_cast<const u32x4 *>(zbase + (size_t)kb_list[k0 + min(i, cnt - 1)] * 512);
#pragma unroll
    for (int i = 0; i < DF_MAXK; ++i) {
      const u32x4 zv = i < cnt ? zr[i] : zero;
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(ur[i][0]), dec_bf16x8(zv), acc0, 0, 0, 0);
      if (nc > 1) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(ur[i][1]), dec_bf16x8(zv), acc1, 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // the stashed operands (each lane reads back what it wrote: no barrier needed)
    if (nstash > 0) {
      u32x4 zs[DF_STASH];
#pragma unroll
      for (int i = 0; i < DF_STASH; ++i)
        zs[i] = *reinterpret_cast<const u32x4 *>(zbase + (size_t)kb_list[k0 + min(DF_MAXK + i, cnt - 1)] * 512);
#pragma unroll
      for (int i = 0; i < DF_STASH; ++i) {
        const u32x4 zv = i < nstash ? zs[i] : zero;
        const u32x4 ua = *reinterpret_cast<const u32x4 *>(my_stash + (i * 2 + 0) * 512);
        const u32x4 ub = *reinterpret_cast<const u32x4 *>(my_stash + (i * 2 + 1) * 512);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(ua), dec_bf16x8(zv), acc0, 0, 0, 0);
        if (nc > 1) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(ub), dec_bf16x8(zv), acc1, 0, 0, 0);
      }
    }
    // anything beyond both budgets is streamed now
    for (int c = DF_MAXK + DF_STASH; c < cnt; c += DEC_CHUNK) {
      u32x4 u0r[DEC_CHUNK], u1r[DEC_CHUNK], zz[DEC_CHUNK];
#pragma unroll
      for (int i = 0; i < DEC_CHUNK; ++i) {
        const int kb = kb_list[k0 + min(c + i, cnt - 1)];
        u0r[i] = *reinterpret_cast<const u32x4 *>(ubase + (size_t)kb * ustep);
        u1r[i] = *reinterpret_cast<const u32x4 *>(ubase + (size_t)kb * ustep + second_off);
        zz[i] = *reinterpret_cast<const u32x4 *>(zbase + (size_t)kb * 512);
      }
#pragma unroll
      for (int i = 0; i < DEC_CHUNK; ++i) {
        const u32x4 zv = (c + i < cnt) ? zz[i] : zero;
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(u0r[i]), dec_bf16x8(zv), acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(u1r[i]), dec_bf16x8(zv), acc1, 0, 0, 0);
      }
    }
  }
  DEC_STAMP(5);
  // per column block: add the wavefronts' contributions in wave order and store
  for (int jl = 0; jl < nc; ++jl) {
#pragma unroll
    for (int e = 0; e < 16; ++e) red[wave][e][lane] = jl == 0 ? acc0[e] : acc1[e];
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
  DEC_STAMP(6);
}

constexpr size_t DF_LDS_A = 32 * DF_XLD * sizeof(uint16_t);
constexpr size_t DF_LDS_D = DF_MAXKB * sizeof(int32_t) + (size_t)DF_WAVES * DF_STASH * 2 * 512 * sizeof(uint16_t);
constexpr size_t DF_LDS_BYTES = DF_WAVES * 16 * 64 * sizeof(float) + (DF_LDS_A > DF_LDS_D ? DF_LDS_A : DF_LDS_D);
static_assert(DF_LDS_BYTES <= 160 * 1024, "LDS budget");

static int g_decode_schedule = 0;   // 0 = one launch when the shape allows, 1 = always three launches
void set_decode_schedule(int v) { g_decode_schedule = v; }

// slices of n in the one-launch form: about one task per workgroup, a slice no longer than DF_MAXSLICE steps
static int persist_slices(int n, int R, int n_wg) {
  const int nkb = n / 16, nquads = (R / 32 + 3) / 4;
  int S = n_wg / nquads;
  const int s_min = (nkb + DF_MAXSLICE - 1) / DF_MAXSLICE;
  if (S < s_min) S = s_min;
  if (S < 1) S = 1;
  if (S > nkb) S = nkb;
  return S;
}
constexpr int DF_MAX_SLICES = 64;   // workspace is sized for this many fp32 partials

static int decode_slices(int R) {
  int ks = (640 + R / 32 - 1) / (R / 32);
  if (ks < 1) ks = 1;
  if (ks > 16) ks = 16;
  return ks;
}

size_t decode_workspace_bytes(const parse_layer *L) {
  const int KS = decode_slices(L->R) > DF_MAX_SLICES ? decode_slices(L->R) : DF_MAX_SLICES;
  return round_up((size_t)KS * 32 * L->R * sizeof(float), 256) + round_up((size_t)L->R * 32 * sizeof(uint16_t), 256) +
         round_up((DEC_MAXG + 1) * sizeof(int32_t), 256);
}

int forward_decode_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *x, int B,
                        const int32_t *pattern_id, uint16_t *y, void *workspace, hipStream_t s) {
  const int gs = L->R / L->G;
  const int KS = decode_slices(L->R);
  const int KSW = KS > DF_MAX_SLICES ? KS : DF_MAX_SLICES;
  static int n_cu = 0;
  static unsigned call_index = 0;
  if (n_cu == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    PARSE_HIP_TRY(hipGetDevice(&dev));
    PARSE_HIP_TRY(hipGetDeviceProperties(&prop, dev));
    n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  float *zp = reinterpret_cast<float *>(workspace);
  uint16_t *zf = reinterpret_cast<uint16_t *>((char *)workspace + round_up((size_t)KSW * 32 * L->R * sizeof(float), 256));
  int32_t *used = reinterpret_cast<int32_t *>((char *)zf + round_up((size_t)L->R * 32 * sizeof(uint16_t), 256));
  const int ncb = L->m / 32;
  const int S = persist_slices(L->n, L->R, n_cu);
  // one launch: a worker takes at most two column blocks, the slices fit the workspace and the LDS stage
  if (g_decode_schedule == 0 && (ncb + n_cu - 1) / n_cu <= 2 && L->R / 16 <= DF_MAXKB && S <= DF_MAX_SLICES &&
      (L->n / 16 + S - 1) / S <= DF_MAXSLICE) {
    static bool attr_done = false;
    if (!attr_done) {
      PARSE_HIP_TRY(hipFuncSetAttribute((const void *)decode_persist, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)DF_LDS_BYTES));
      attr_done = true;
    }
    DfArgs a{(const uint16_t *)L->Vt, (const uint16_t *)L->Ut, x, y, zf, zp, pt->subsets, pattern_id, pt->subset_stride,
             pt->k, pt->n_patterns, B, L->n, L->m, L->R, L->G, gs, S, (int)(call_index++ % DF_SLOTS),
             (long long *)(zp + (size_t)(DF_MAX_SLICES - 1) * 32 * L->R)};   // diagnostics only: the last, unused slice
    void *params[] = {&a};
    PARSE_HIP_TRY(hipLaunchCooperativeKernel((const void *)decode_persist, dim3(n_cu), dim3(DF_THREADS), params,
                                             (unsigned)DF_LDS_BYTES, s));
    return PARSE_OK;
  }
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
