// a7: decode step for bf16 PARSE_MFMA16 layers (Sec. 4.3, "Rank Reuse for Decoding"): every sequence keeps the
// rank subset chosen at prefill; one token per sequence.  Bandwidth-bound: the kernels stream each rank group
// that ANY sequence of the batch selected exactly once, straight from the layer's factor store in operand
// order (1 KiB coalesced per wavefront instruction, no LDS hop, no packed copies), and apply it to all
// sequences at once on the matrix cores (32 sequences = the N side of a 32x32x16 instruction).  A sequence
// whose pattern does not hold a group gets a zero in that group's part of z, so it contributes nothing.
// Three launches: decode_z (Vt stream -> fp32 partials of z per slice of n), decode_zfin (tiny: adds the slices
// up in slice order, masks, rounds, operand order), decode_y (Ut stream -> y).  A compute unit sustains only
// about 50 GB/s of cache-line fills, so both streams are cut into about as many workgroups as there are units,
// and the small operands (x, z) are shared inside a workgroup instead of being re-fetched per factor operand.
// The streaming loops are branch-free: operand lists are walked in chunks with fetches past the end clamped
// to the last valid operand and their contribution switched off by zeroing the small operand.
// Horizontal fusion (Sec. 4.4, Eq. 11-12): up to DEC_MAX_LAYERS layers that read the SAME x (Q/K/V, gate/up)
// go through the same three launches together -- each launch's grid is the concatenation of the layers' task
// lists, so the per-launch floor is paid once and x is staged once per task whichever layer the task belongs to.
#include "common.hpp"

namespace parse {

constexpr int DZ_WAVES = 8, DZ_THREADS = DZ_WAVES * 64;
constexpr int DY_WAVES = 8, DY_THREADS = DY_WAVES * 64;
constexpr int DEC_CHUNK = 4;       // operands fetched per chunk; four chunks in flight per wavefront
constexpr int DEC_MAXG = 64;
constexpr int DZ_MAXSLICE = 64;    // reduction steps (of 16 columns) of x staged per decode_z task
constexpr int DZ_XLD = DZ_MAXSLICE * 16 + 8;
constexpr int DEC_MAX_SLICES = 64; // slices of n the workspace is sized for
constexpr int DY_CHUNK = 4;        // decode_y: operands per chunk after the first block
constexpr int DY_MAXKB = 1024;     // selected reduction blocks a decode_y workgroup can list

constexpr int DEC_MAX_LAYERS = 4;

struct DecLayer {
  const uint16_t *Vt, *Ut;
  uint16_t *y;
  const int32_t *subsets;      // this layer's patterns
  int stride, k, n_patterns;
  float *zp;                   // workspace parts of this layer
  uint16_t *zf;
  int32_t *used;
  int R, G, gs, m;
  int z_first, f_first, y_first;   // first workgroup of this layer in decode_z / decode_zfin / decode_y
};
struct DecArgs {
  DecLayer L[DEC_MAX_LAYERS];
  int n_layers;
  const uint16_t *x;
  const int32_t *pattern_id;
  int B, n, S;                 // sequences, input width, slices of n (the same for every layer)
};

__device__ __forceinline__ bf16x8 dec_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

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

// ---------------------------------------------------------------------------------------------------------
// decode_z: z partials.  grid = nquads * S tasks; task = (four consecutive 32-rank blocks, slice s of n).
// The slice of the token rows x is staged in LDS once (coalesced row reads; the matrix-core operand read
// pattern is only ever applied to LDS) and shared by the four rank blocks; wavefront w owns rank block w % 4
// and half w / 4 of the slice; its Vt operands come straight from the store, four chunks in flight; the two
// halves add up through LDS; fp32 partials go to the workspace as zp[quad][slice][piece][8], a piece being the
// 8 ranks x 1 sequence that one lane of the next product holds, so that both this kernel's stores and
// decode_zfin's loads are contiguous per wavefront.  Rank blocks of groups nobody selected are skipped (nothing
// of them is read or written).  Workgroup 0 also lists the groups selected by at least one sequence
// (ascending) for decode_y.
__global__ __launch_bounds__(DZ_THREADS) void decode_z(DecArgs a) {
  int li = 0;
#pragma unroll
  for (int i = 1; i < DEC_MAX_LAYERS; ++i) li += (i < a.n_layers && (int)blockIdx.x >= a.L[i].z_first) ? 1 : 0;
  const DecLayer &ly = a.L[li];
  const uint16_t *__restrict__ Vt = ly.Vt;
  const uint16_t *__restrict__ x = a.x;
  const int32_t *__restrict__ subsets = ly.subsets;
  const int32_t *__restrict__ pattern_id = a.pattern_id;
  float *__restrict__ zp = ly.zp;
  int32_t *__restrict__ used_out = ly.used;   // [0] = count, [1..] = ids
  const int B = a.B, n = a.n, R = ly.R, G = ly.G, gs = ly.gs, stride = ly.stride, k = ly.k, n_patterns = ly.n_patterns;
  const int S = a.S;
  const int bid = blockIdx.x - ly.z_first;    // task within the layer
  __shared__ __attribute__((aligned(16))) uint16_t xs[32 * DZ_XLD];  // 66 KiB; reused for the halves' sum
  __shared__ uint32_t gmask[DEC_MAXG];
  float(*red)[16][64] = reinterpret_cast<float(*)[16][64]>(xs);       // [4][16][64] floats = 16 KiB
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, q = lane >> 5;
  const int nkb = n / 16, nrb = R / 32;
  const int quad = bid / S, sl = bid - quad * S;
  const int w0 = (int)(((long long)nkb * sl) / S), w1 = (int)(((long long)nkb * (sl + 1)) / S);
  const int len = w1 - w0;                                           // <= DZ_MAXSLICE (host)
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int rbl = wave_s & 3, half = wave_s >> 2;
  const int rb = quad * 4 + rbl;
  const int h0 = (len * half) / 2, h1 = (len * (half + 1)) / 2;      // this wavefront's steps of the slice
  const int cnt_all = rb < nrb ? h1 - h0 : 0;
  const char *vblock = reinterpret_cast<const char *>(Vt) + ((size_t)min(rb, nrb - 1) * nkb + w0 + h0) * 1024;
  const uint32_t lane_off = lane * 16;
  u32x4 V0[DEC_CHUNK], V1[DEC_CHUNK], V2[DEC_CHUNK], V3[DEC_CHUNK];
  auto load_v = [&](u32x4 *V, int base, int cnt) {
#pragma unroll
    for (int i = 0; i < DEC_CHUNK; ++i)
      V[i] = *reinterpret_cast<const u32x4 *>(vblock + (size_t)max(min(base + i, cnt - 1), 0) * 1024 + lane_off);
  };
  // x slice: rows of len*32 bytes in 16-byte pieces; all of a lane's pieces (at most 8) are requested together
  const int ppr = len * 2;
  u32x4 xp[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int piece = min(i * DZ_THREADS + (int)threadIdx.x, 32 * ppr - 1);
    const int r = piece / ppr, c = (piece - r * ppr) * 8;
    xp[i] = *reinterpret_cast<const u32x4 *>(x + (size_t)min(r, B - 1) * n + (size_t)w0 * 16 + c);
  }
  if (threadIdx.x < DEC_MAXG) gmask[threadIdx.x] = 0;
  __syncthreads();
  build_group_masks(subsets, stride, k, n_patterns, pattern_id, B, G, gmask);
  if (bid == 0 && threadIdx.x < 64) {
    const bool u = lane < G && gmask[lane] != 0u;
    const unsigned long long mask = __ballot(u);
    if (u) used_out[1 + __popcll(mask & ((1ull << lane) - 1ull))] = lane;
    if (lane == 0) used_out[0] = __popcll(mask);
  }
  bool any = false;
  for (int i = 0; i < 4; ++i) {
    const int r = quad * 4 + i;
    any = any || (r < nrb && gmask[r * 32 / gs] != 0u);
  }
  if (!any) return;   // uniform: nobody selected any of these rank blocks
  const bool live = rb < nrb && gmask[min(rb, nrb - 1) * 32 / gs] != 0u;   // uniform per wavefront
  const int cnt = live ? cnt_all : 0;
  load_v(V0, 0, cnt);
  load_v(V1, DEC_CHUNK, cnt);
  load_v(V2, 2 * DEC_CHUNK, cnt);
  load_v(V3, 3 * DEC_CHUNK, cnt);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int piece = i * DZ_THREADS + threadIdx.x;
    if (piece < 32 * ppr) {
      const int r = piece / ppr, c = (piece - r * ppr) * 8;
      *reinterpret_cast<u32x4 *>(xs + r * DZ_XLD + c) = r < B ? xp[i] : u32x4{0, 0, 0, 0};
    }
  }
  __syncthreads();      // x slice staged
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  const uint16_t *xb_base = xs + l32 * DZ_XLD + h0 * 16 + q * 8;
  const u32x4 zero = {0, 0, 0, 0};
  auto compute = [&](const u32x4 *V, int base) {
#pragma unroll
    for (int i = 0; i < DEC_CHUNK; ++i) {
      const int st = min(base + i, max(cnt - 1, 0));
      const u32x4 xv = *reinterpret_cast<const u32x4 *>(xb_base + st * 16);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(V[i]), dec_bf16x8(base + i < cnt ? xv : zero), acc, 0, 0, 0);
    }
  };
  for (int c0 = 0; c0 < cnt; c0 += 4 * DEC_CHUNK) {
    compute(V0, c0);
    __builtin_amdgcn_sched_barrier(0);
    load_v(V0, c0 + 4 * DEC_CHUNK, cnt);
    __builtin_amdgcn_sched_barrier(0);
    compute(V1, c0 + DEC_CHUNK);
    __builtin_amdgcn_sched_barrier(0);
    load_v(V1, c0 + 5 * DEC_CHUNK, cnt);
    __builtin_amdgcn_sched_barrier(0);
    compute(V2, c0 + 2 * DEC_CHUNK);
    __builtin_amdgcn_sched_barrier(0);
    load_v(V2, c0 + 6 * DEC_CHUNK, cnt);
    __builtin_amdgcn_sched_barrier(0);
    compute(V3, c0 + 3 * DEC_CHUNK);
    __builtin_amdgcn_sched_barrier(0);
    load_v(V3, c0 + 7 * DEC_CHUNK, cnt);
    __builtin_amdgcn_sched_barrier(0);
  }
  __syncthreads();      // every wavefront is done with the x slice; its LDS now holds the halves' sum
  if (half == 1) {
#pragma unroll
    for (int e = 0; e < 16; ++e) red[rbl][e][lane] = acc[e];
  }
  __syncthreads();
  float *zq = zp + (size_t)quad * S * 4096;   // this quad's partials: [S][512 pieces][8]
  if (half == 0 && live) {
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] += red[rbl][e][lane];
    // entries of sequences whose pattern does not hold the rank's group are zero in z
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      const bool member = (gmask[(rb * 32 + 8 * blk + 4 * q) / gs] >> l32) & 1u;
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[blk * 4 + j] = member ? acc[blk * 4 + j] : 0.f;
    }
    // lane: sequence l32, local ranks rbl*32 + 8*blk + 4*q + (0..3) = piece (rbl*4 + blk)*32 + l32, floats 4q..4q+3
    float *dst = zq + (size_t)sl * 4096 + ((rbl * 4) * 32 + l32) * 8 + q * 4;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
      *reinterpret_cast<float4 *>(dst + blk * 256) = float4{acc[blk * 4], acc[blk * 4 + 1], acc[blk * 4 + 2], acc[blk * 4 + 3]};
  }
}

// ---------------------------------------------------------------------------------------------------------
// decode_zfin: z = sum of the S slices (in slice order), rounded to bf16, stored in operand order: piece
// o = (kb*2 + q)*32 + b holds z[b][16kb + 8q + (0..7)] (the partials use the same piece numbering and are
// already masked).  One wavefront per workgroup, one piece per lane, the loads of eight slices in flight at
// once.  Pieces of rank blocks nobody selected hold whatever the workspace held; decode_y never reads them.
__global__ __launch_bounds__(64) void decode_zfin(DecArgs a) {
  int li = 0;
#pragma unroll
  for (int i = 1; i < DEC_MAX_LAYERS; ++i) li += (i < a.n_layers && (int)blockIdx.x >= a.L[i].f_first) ? 1 : 0;
  const DecLayer &ly = a.L[li];
  const float *__restrict__ zp = ly.zp;
  uint16_t *__restrict__ zf = ly.zf;
  const int S = a.S, R = ly.R;
  const int o = ((int)blockIdx.x - ly.f_first) * 64 + threadIdx.x;   // piece
  const int quad = o >> 9, t = o & 511;
  if ((o >> 5) * 8 >= R) return;
  float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const float *src = zp + ((size_t)quad * S * 512 + t) * 8;
#pragma unroll 8
  for (int s2 = 0; s2 < S; ++s2) {
    const float4 f0 = *reinterpret_cast<const float4 *>(src + (size_t)s2 * 4096);
    const float4 f1 = *reinterpret_cast<const float4 *>(src + (size_t)s2 * 4096 + 4);
    v[0] += f0.x; v[1] += f0.y; v[2] += f0.z; v[3] += f0.w;
    v[4] += f1.x; v[5] += f1.y; v[6] += f1.z; v[7] += f1.w;
  }
  u32x4 w;
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(v[2 * e], v[2 * e + 1]);
  *reinterpret_cast<u32x4 *>(zf + (size_t)o * 8) = w;
}

// ---------------------------------------------------------------------------------------------------------
// decode_y: y.  grid = ceil(ncb / NC) workgroups, each owns NC (1 or 2) consecutive 32-column output blocks;
// wavefront w owns an eighth of the selected reduction blocks for all NC column blocks, so one z operand
// (cache-resident) feeds NC products; the Ut operands of its first MAXK reduction blocks are requested at
// once (MAXK sized so that everything stays in registers), the rest is streamed in chunks; the eight wavefronts
// add up through LDS.
template <int NC>
__global__ __launch_bounds__(DY_THREADS) void decode_y(DecArgs a) {
  int li = 0;
#pragma unroll
  for (int i = 1; i < DEC_MAX_LAYERS; ++i) li += (i < a.n_layers && (int)blockIdx.x >= a.L[i].y_first) ? 1 : 0;
  const DecLayer &ly = a.L[li];
  const uint16_t *__restrict__ Ut = ly.Ut;
  const uint16_t *__restrict__ zf = ly.zf;
  const int32_t *__restrict__ used_in = ly.used;
  uint16_t *__restrict__ y = ly.y;
  const int B = a.B, m = ly.m, G = ly.G, gs = ly.gs;
  const int bid = blockIdx.x - ly.y_first;
  __shared__ float red[DY_WAVES][16][64];
  __shared__ int32_t kb_list[DY_MAXKB];
  __shared__ int32_t used[DEC_MAXG];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, q = lane >> 5;
  const int ncb = m / 32;
  const int c0 = bid * NC;
  const int nc = min(NC, ncb - c0);
  // count and ids are fetched together (ids past the count are whatever the list held; they are not used)
  const int n_used_raw = used_in[0];
  if (threadIdx.x < DEC_MAXG) used[threadIdx.x] = used_in[1 + threadIdx.x];
  const int n_used = max(0, min(n_used_raw, G));
  __syncthreads();
  const int kpg = gs / 16;                 // reduction blocks per group
  const int total_kb = n_used * kpg;       // selected reduction blocks
  for (int i = threadIdx.x; i < total_kb; i += DY_THREADS) kb_list[i] = used[i / kpg] * kpg + i % kpg;
  __syncthreads();
  const int k0 = (total_kb * wave) / DY_WAVES, k1 = (total_kb * (wave + 1)) / DY_WAVES;
  const int cnt = k1 - k0;
  const uint16_t *ubase = Ut + ((size_t)c0 * 64 + lane) * 8;
  const uint16_t *zbase = zf + (size_t)lane * 8;
  const size_t ustep = (size_t)ncb * 512;
  int coff[NC];   // element offset of column block j's operand; blocks past the end re-read block 0 (result unused)
#pragma unroll
  for (int j = 0; j < NC; ++j) coff[j] = j < nc ? j * 512 : 0;
  f32x16 acc[NC];
#pragma unroll
  for (int j = 0; j < NC; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  const u32x4 zero = {0, 0, 0, 0};
  constexpr int DY_MAXK = NC == 1 ? 20 : (NC == 2 ? 16 : (NC == 3 ? 12 : 8));
  constexpr int DEC_CHUNK = DY_CHUNK;
  if (cnt > 0) {
    u32x4 ur[DY_MAXK][NC], zr[DY_MAXK];
#pragma unroll
    for (int i = 0; i < DY_MAXK; ++i) {
      const int kb = kb_list[k0 + min(i, cnt - 1)];
#pragma unroll
      for (int j = 0; j < NC; ++j) ur[i][j] = *reinterpret_cast<const u32x4 *>(ubase + (size_t)kb * ustep + coff[j]);
      zr[i] = *reinterpret_cast<const u32x4 *>(zbase + (size_t)kb * 512);
    }
    __builtin_amdgcn_sched_barrier(0);   // every fetch above is in flight before the first product
#pragma unroll
    for (int i = 0; i < DY_MAXK; ++i) {
      const u32x4 zv = i < cnt ? zr[i] : zero;
#pragma unroll
      for (int j = 0; j < NC; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(ur[i][j]), dec_bf16x8(zv), acc[j], 0, 0, 0);
    }
    for (int c = DY_MAXK; c < cnt; c += DEC_CHUNK) {
      u32x4 uu[DEC_CHUNK][NC], zz[DEC_CHUNK];
#pragma unroll
      for (int i = 0; i < DEC_CHUNK; ++i) {
        const int kb = kb_list[k0 + min(c + i, cnt - 1)];
#pragma unroll
        for (int j = 0; j < NC; ++j) uu[i][j] = *reinterpret_cast<const u32x4 *>(ubase + (size_t)kb * ustep + coff[j]);
        zz[i] = *reinterpret_cast<const u32x4 *>(zbase + (size_t)kb * 512);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < DEC_CHUNK; ++i) {
        const u32x4 zv = (c + i < cnt) ? zz[i] : zero;
#pragma unroll
        for (int j = 0; j < NC; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(uu[i][j]), dec_bf16x8(zv), acc[j], 0, 0, 0);
      }
    }
  }
  // per column block: add the wavefronts' contributions in wave order and store
#pragma unroll
  for (int jl = 0; jl < NC; ++jl) {
    if (jl < nc) {   // uniform
#pragma unroll
      for (int e = 0; e < 16; ++e) red[wave][e][lane] = acc[jl][e];
      __syncthreads();
      for (int i = threadIdx.x; i < 16 * 64; i += DY_THREADS) {
        const int e = i >> 6, ln = i & 63;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < DY_WAVES; ++w) sum += red[w][e][ln];
        red[0][e][ln] = sum;   // each (e, ln) is read and written by this thread only
      }
      __syncthreads();
      if (wave == 0 && l32 < B) {
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
          u32x2 w;
          w[0] = pack_bf16x2(red[0][blk * 4 + 0][lane], red[0][blk * 4 + 1][lane]);
          w[1] = pack_bf16x2(red[0][blk * 4 + 2][lane], red[0][blk * 4 + 3][lane]);
          *reinterpret_cast<u32x2 *>(y + (size_t)l32 * m + (c0 + jl) * 32 + blk * 8 + q * 4) = w;
        }
      }
      __syncthreads();
    }
  }
}

// Slices of n: at most one task per compute unit over the rank quads (of all layers of the call) that can be
// selected at all (the host knows k and the number of patterns, not the subsets), a slice no longer than
// DZ_MAXSLICE steps, at most DEC_MAX_SLICES slices.
static int live_quads_bound(const parse_layer *L, const parse_patterns *pt) {
  const int gs = L->R / L->G, nquads = (L->R / 32 + 3) / 4;
  long long groups = (long long)pt->k * pt->n_patterns;
  if (groups > L->G) groups = L->G;
  long long live = (groups * gs + 127) / 128;
  if (live > nquads) live = nquads;
  return live < 1 ? 1 : (int)live;
}

static int decode_slices(int n, int live, int n_cu) {
  const int nkb = n / 16;
  int S = n_cu / live;   // rounded down: a unit that gets two tasks runs both at half the rate
  const int s_min = (nkb + DZ_MAXSLICE - 1) / DZ_MAXSLICE;
  if (S < s_min) S = s_min;
  if (S > DEC_MAX_SLICES) S = DEC_MAX_SLICES;   // decode_supported() keeps the slice within DZ_MAXSLICE
  if (S > nkb) S = nkb;
  if (S < 1) S = 1;
  return S;
}

static size_t dec_zp_bytes(const parse_layer *L) {
  const int nquads = (L->R / 32 + 3) / 4;
  return round_up((size_t)DEC_MAX_SLICES * nquads * 4096 * sizeof(float), 256);
}
static size_t dec_zf_bytes(const parse_layer *L) {
  const int nquads = (L->R / 32 + 3) / 4;
  return round_up((size_t)nquads * 4096 * sizeof(uint16_t), 256);
}

size_t decode_workspace_bytes(const parse_layer *L) {
  return dec_zp_bytes(L) + dec_zf_bytes(L) + round_up((DEC_MAXG + 1) * sizeof(int32_t), 256);
}

bool decode_supported(const parse_layer *L) {
  const int s_min = (L->n / 16 + DZ_MAXSLICE - 1) / DZ_MAXSLICE;
  return s_min <= DEC_MAX_SLICES && L->R / 16 <= DY_MAXKB && L->G <= DEC_MAXG;
}

// n_layers layers that share x (same n); Y[l] and the workspace part of layer l follow the order of `layers`.
int forward_decode_multi_bf16(const parse_layer *layers, const parse_patterns *pts, int n_layers, const uint16_t *x,
                              int B, const int32_t *pattern_id, uint16_t *const *Y, void *workspace, hipStream_t s) {
  if (n_layers < 1 || n_layers > DEC_MAX_LAYERS) return PARSE_ESHAPE;
  static int n_cu_of[64] = {0};
  int dev = 0;
  PARSE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return PARSE_EINVAL;
  if (n_cu_of[dev] == 0) {
    hipDeviceProp_t prop;
    PARSE_HIP_TRY(hipGetDeviceProperties(&prop, dev));
    n_cu_of[dev] = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  const int n_cu = n_cu_of[dev];
  DecArgs a{};
  a.n_layers = n_layers;
  a.x = x;
  a.pattern_id = pattern_id;
  a.B = B;
  a.n = layers[0].n;
  int live = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (!decode_supported(&layers[l])) return PARSE_ESHAPE;
    if (layers[l].n != a.n) return PARSE_ESHAPE;
    live += live_quads_bound(&layers[l], &pts[l]);
  }
  a.S = decode_slices(a.n, live, n_cu);
  // column blocks per workgroup (one z operand feeds NC products): the smallest count that puts at most one
  // workgroup on a compute unit -- a unit with two streams at half the rate and sets the kernel's time
  int NC = 1;
  for (; NC < 4; ++NC) {
    int wgs = 0;
    for (int l = 0; l < n_layers; ++l) wgs += (layers[l].m / 32 + NC - 1) / NC;
    if (wgs <= n_cu) break;
  }
  char *ws = reinterpret_cast<char *>(workspace);
  int zb = 0, fb = 0, yb = 0;
  for (int l = 0; l < n_layers; ++l) {
    const parse_layer *L = &layers[l];
    DecLayer &d = a.L[l];
    d.Vt = (const uint16_t *)L->Vt;
    d.Ut = (const uint16_t *)L->Ut;
    d.y = Y[l];
    d.subsets = pts[l].subsets;
    d.stride = pts[l].subset_stride;
    d.k = pts[l].k;
    d.n_patterns = pts[l].n_patterns;
    d.zp = reinterpret_cast<float *>(ws);
    d.zf = reinterpret_cast<uint16_t *>(ws + dec_zp_bytes(L));
    d.used = reinterpret_cast<int32_t *>(ws + dec_zp_bytes(L) + dec_zf_bytes(L));
    ws += decode_workspace_bytes(L);
    d.R = L->R; d.G = L->G; d.gs = L->R / L->G; d.m = L->m;
    const int nquads = (L->R / 32 + 3) / 4, ncb = L->m / 32;
    d.z_first = zb; zb += nquads * a.S;
    d.f_first = fb; fb += nquads * 8;
    d.y_first = yb; yb += (ncb + NC - 1) / NC;
  }
  hipLaunchKernelGGL(decode_z, dim3(zb), dim3(DZ_THREADS), 0, s, a);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(decode_zfin, dim3(fb), dim3(64), 0, s, a);
  PARSE_LAUNCH_CHECK();
  if (NC == 1) hipLaunchKernelGGL(decode_y<1>, dim3(yb), dim3(DY_THREADS), 0, s, a);
  else if (NC == 2) hipLaunchKernelGGL(decode_y<2>, dim3(yb), dim3(DY_THREADS), 0, s, a);
  else if (NC == 3) hipLaunchKernelGGL(decode_y<3>, dim3(yb), dim3(DY_THREADS), 0, s, a);
  else hipLaunchKernelGGL(decode_y<4>, dim3(yb), dim3(DY_THREADS), 0, s, a);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

int forward_decode_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *x, int B,
                        const int32_t *pattern_id, uint16_t *y, void *workspace, hipStream_t s) {
  uint16_t *Y[1] = {y};
  return forward_decode_multi_bf16(L, pt, 1, x, B, pattern_id, Y, workspace, s);
}

}  // namespace parse
