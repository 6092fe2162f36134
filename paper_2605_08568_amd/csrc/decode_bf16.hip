// a7: decode step for bf16 PARSE_MFMA16 layers (Sec. 4.3, "Rank Reuse for Decoding"): every sequence keeps the
// rank subset chosen at prefill; one token per sequence.  Bandwidth-bound: the kernels stream each rank group that
// ANY sequence of the batch selected exactly once, straight from the layer's factor store in operand order
// (1 KiB coalesced per wavefront instruction, no packed copies), and apply it to all sequences at once on the
// matrix cores (32 sequences = the N side of a 32x32x16 instruction).  A sequence whose pattern does not hold a
// group gets a zero in that group's part of z, so it contributes nothing.
//
// Decode plan (Sec. 4.3: the subsets are fixed after prefill, so everything derived from them is computed once per
// batch, not once per step): per layer the sequence mask of every group, the ascending list of groups selected by at
// least one sequence and their count, plus the arrival counters of decode_zr's split reduction.  decode_plan_build
// writes it; the kernels below read it (decode_zr also draws and resets its tickets there).
//
// Two launches per step:
//   decode_zr  one workgroup per 32-rank block of a used group (operand-order layers have groups of whole blocks) and slice
//              of the reduction range: the Vt operands go straight into registers, all of a wavefront's at once; the x
//              rows of the slice are staged in LDS; long reductions are cut in slices whose partial sums the last
//              workgroup of a ticket adds in slice order.  z ends up masked, rounded to bf16 and stored as operands of
//              the second product.
//   decode_y   NC (1..4) 32-column output blocks per workgroup; the eight wavefronts split the used reduction blocks,
//              all Ut operands requested up front; LDS reduction in wavefront order.
// A handful of sequences (B <= 4) take decode_zv / decode_yv instead: the same two products on the vector units with a
// finer split of the work (eight ranks, sixteen or thirty-two columns per workgroup), because one to four sequences
// leave the matrix instruction's 32-wide N side and most 32-rank workgroups idle.
// Horizontal fusion (Sec. 4.4, Eq. 11-12): up to DEC_MAX_LAYERS layers that read the SAME x (Q/K/V, gate/up) go
// through the same two launches together -- each launch's grid is the concatenation of the layers' task lists.
// No floating-point atomics; the summation order is fixed: same inputs, same bits.
#include <algorithm>

#include "prefill_common.hpp"

namespace parse {

constexpr int DY_WAVES = 8, DY_THREADS = DY_WAVES * 64;
constexpr int DEC_MAXG = 64;
constexpr int DY_CHUNK = 4;                // decode_y: operands per chunk after the first block
constexpr int DY_MAXKB = 1024;             // selected reduction blocks a decode_y workgroup can list
constexpr int DEC_MAX_LAYERS = 4;
constexpr int DEC_TICKETS = 512;           // 32-rank blocks of the largest layer (R = 16384)
constexpr int DEC_PLAN_WORDS = 192 + DEC_TICKETS;   // per layer: [0] count, [1..64] used group ids, [65..128] sequence masks,
                                                    // [192..) arrival counters of the split reduction (zero between calls)

#define PARSE_DEC_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define PARSE_DEC_GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

struct DecLayer {
  const uint16_t *Vt, *Ut;
  uint16_t *y;
  uint16_t *zf;                // workspace: z of this layer in operand order
  const int32_t *plan;         // this layer's DEC_PLAN_WORDS of the decode plan
  float *zpart;                // workspace: partial sums of z, [R/32][KS][16][64] floats (KS > 1)
  int32_t *ticket;             // [DEC_TICKETS] arrival counters in the plan, one per 32-rank block
  int R, G, gs, m;
  int z_first, y_first;        // first workgroup of this layer in decode_zr / decode_y
};
struct DecArgs {
  DecLayer L[DEC_MAX_LAYERS];
  int n_layers;
  const uint16_t *x;
  int B, n;
  int KS;                      // decode_zr: slices of the reduction range
};

struct DecPlanArgs {
  const int32_t *subsets[DEC_MAX_LAYERS];
  int stride[DEC_MAX_LAYERS], k[DEC_MAX_LAYERS], n_patterns[DEC_MAX_LAYERS], G[DEC_MAX_LAYERS];
  const int32_t *pattern_id;
  int B;
  int32_t *plan;
};

__device__ __forceinline__ bf16x8 dec_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// grid = layers, one wavefront each: lane b < B looks at its sequence's k group ids and ORs its bit into the groups'
// masks (LDS, integer OR: order-free); then the used groups are listed in ascending order by a vote.
__global__ __launch_bounds__(64) void decode_plan_build(DecPlanArgs a) {
  __shared__ uint32_t gmask[DEC_MAXG];
  const int l = blockIdx.x, lane = threadIdx.x;
  int32_t *out = a.plan + (size_t)l * DEC_PLAN_WORDS;
  gmask[lane] = 0u;
  __syncthreads();
  const int G = a.G[l];
  if (lane < a.B && lane < 32) {
    const int pid = a.pattern_id[lane];
    if (pid >= 0 && pid < a.n_patterns[l]) {
      for (int i = 0; i < a.k[l]; ++i) {
        const int g = a.subsets[l][(size_t)pid * a.stride[l] + i];
        if (g >= 0 && g < G) atomicOr(&gmask[g], 1u << lane);
      }
    }
  }
  __syncthreads();
  __shared__ int32_t used_l[DEC_MAXG];
  const bool u = lane < G && gmask[lane] != 0u;
  const unsigned long long votes = __ballot(u);
  used_l[lane] = -1;
  __syncthreads();
  if (u) used_l[__popcll(votes & ((1ull << lane) - 1ull))] = lane;
  __syncthreads();
  out[1 + lane] = used_l[lane];
  out[65 + lane] = (int32_t)gmask[lane];
  if (lane == 0) out[0] = __popcll(votes);
  for (int i = lane; i < DEC_TICKETS; i += 64) out[192 + i] = 0;
}

// ---------------------------------------------------------------------------------------------------------
// decode_zr.  Workgroup = (layer, 32-rank block, slice s of KS of the reduction range).  A slice is at most 256 reduction steps (4096 columns): each of the eight wavefronts
// owns an eighth of it and requests ALL its Vt operands at once, straight into registers (1 KiB coalesced per
// instruction, up to 32 of them): the registers of the eight wavefronts are the staging buffer -- 256 KiB of factor
// stream in flight per compute unit, several times what LDS staging can hold, which is what a stream from HBM needs.
// The x rows of the slice are staged in LDS (loads that write LDS directly; 512-byte row segments, 16-byte pieces
// XOR-swizzled by the row so that an operand read -- 32 rows x the same piece -- spreads over the banks), at most 128
// steps at a time.  TWO == false (slices of up to 128 steps): one wait, one barrier, then the products run from registers
// and LDS.  TWO == true: the slice is staged in two halves; a wavefront's operands are ordered first half, second half,
// so the products of the first half run while the second half of the factor stream is still arriving, and the second
// half of x -- requested as soon as the first is consumed, long before the stream ends -- is there when it does.
// The eight wavefronts' sums are added in wavefront order through LDS.
// KS == 1: the block's z is masked, rounded to bf16 and stored as operands of the second product.
// KS  > 1: the workgroup stores its partial sum (fp32) and takes a ticket of its rank block; the workgroup that draws
// the last ticket adds the KS partial sums in slice order (not in arrival order: same inputs, same bits) and stores the
// operands.  Nobody waits for anybody: a workgroup that is not the last simply ends.  The tickets live in the decode plan
// (zeroed when the plan is built, reset by the last workgroup), so a plan serves one decode call at a time.
constexpr int DR_WAVES = 8, DR_THREADS = DR_WAVES * 64;
constexpr int DR_MAXK = 32;                  // Vt operands a wavefront requests (its eighth of the slice)
constexpr int DR_SEG_KB = 16;                // reduction steps per staged x segment (256 columns, 512 bytes per row)
constexpr int DR_SEG_BYTES = 32 * 512;       // 16 KiB
constexpr int DR_MAXSEG = 8;                 // segments staged at a time: 128 steps, 128 KiB
constexpr int DR_HALF_KB = DR_MAXSEG * DR_SEG_KB;    // 128
constexpr int DR_MAX_KS = 16;
constexpr int DR_TARGET_WGS = 240;           // workgroups wanted per launch: a little under one per compute unit

// lane (j, q) holds s[e] = ranks 8*(e/4) + 4*q + e%4 of sequence j of a 32-rank block: mask, round, pair the bands into
// 8 consecutive ranks and store the two z operands (reduction blocks rb*2, rb*2+1 of the second product)
__device__ __forceinline__ void dec_store_z_operands(const float (&s)[16], uint32_t mask, int lane, uint16_t *zf, int rb) {
  const bool member = (mask >> (lane & 31)) & 1u;     // a sequence outside the group's mask gets zeros
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t p0x = member ? cvt_pk_bf16(s[(2 * h) * 4 + 0], s[(2 * h) * 4 + 1]) : 0u;
    const uint32_t p0y = member ? cvt_pk_bf16(s[(2 * h) * 4 + 2], s[(2 * h) * 4 + 3]) : 0u;
    const uint32_t p1x = member ? cvt_pk_bf16(s[(2 * h + 1) * 4 + 0], s[(2 * h + 1) * 4 + 1]) : 0u;
    const uint32_t p1y = member ? cvt_pk_bf16(s[(2 * h + 1) * 4 + 2], s[(2 * h + 1) * 4 + 3]) : 0u;
    // after the swap lane (j, q) holds the 8 consecutive ranks rb*32 + 16h + 8q + (0..7) of sequence j
    const u32x2 sx = __builtin_amdgcn_permlane32_swap(p0x, p1x, false, false);
    const u32x2 sy = __builtin_amdgcn_permlane32_swap(p0y, p1y, false, false);
    *reinterpret_cast<u32x4 *>((char *)zf + (size_t)(rb * 2 + h) * 1024 + lane * 16) = u32x4{sx[0], sy[0], sx[1], sy[1]};
  }
}

template <bool TWO>
__global__ __launch_bounds__(DR_THREADS) void decode_zr(DecArgs a) {
  constexpr int HK = DR_MAXK / 2;            // TWO: operands per half and wavefront
  int li = 0;
#pragma unroll
  for (int i = 1; i < DEC_MAX_LAYERS; ++i) li += (i < a.n_layers && (int)blockIdx.x >= a.L[i].z_first) ? 1 : 0;
  const DecLayer &ly = a.L[li];
  const int KS = a.KS;
  const int bid = blockIdx.x - ly.z_first;
  const int rb = bid / KS, sl = bid % KS;
  const int n = a.n, B = a.B, gs = ly.gs;
  // sequences whose pattern holds this block's group; a block nobody selected is neither read nor written
  const uint32_t mask = (uint32_t)ly.plan[65 + (rb * 32) / gs];
  if (mask == 0u) return;
  __shared__ __attribute__((aligned(1024))) char xs[DR_MAXSEG * DR_SEG_BYTES];
  __shared__ int32_t am_last;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int j = lane & 31, q = lane >> 5;
  const int nkb = n / 16;
  const int ks0 = (int)(((long long)nkb * sl) / KS), ks1 = (int)(((long long)nkb * (sl + 1)) / KS);
  const int cnt_wg = ks1 - ks0;                         // <= 8 * DR_MAXK, and <= DR_HALF_KB unless TWO (the host picks KS so)
  // the slice in one part (A) or two (A, B); x segments are counted from the start of the slice
  const int nseg = (cnt_wg + DR_SEG_KB - 1) / DR_SEG_KB;
  const int nsegA = TWO ? (nseg + 1) / 2 : nseg;        // <= DR_MAXSEG
  const int cntA = min(cnt_wg, nsegA * DR_SEG_KB), cntB = cnt_wg - cntA;
  const int a0 = (cntA * wave) / DR_WAVES, cntAw = (cntA * (wave + 1)) / DR_WAVES - a0;   // this wavefront's steps of part A
  const int b0 = (cntB * wave) / DR_WAVES, cntBw = (cntB * (wave + 1)) / DR_WAVES - b0;   // ... of part B (<= HK each if TWO)
  const int last_piece = n / 8 - 1;
  // x segments [s0, s0 + ns) of the slice into LDS slots 0..ns-1: a segment is 16 instructions of 1 KiB (two rows of 512
  // bytes each).  Lane l writes slot l % 32 of row 2*ins + l / 32 and fetches the piece (slot ^ (row & 15)) of that row's
  // segment; pieces past the end of the row re-read its last one (their products are switched off below)
  auto stage_x = [&](int s0, int ns) {
#pragma unroll
    for (int u = 0; u < DR_MAXSEG * 16 / DR_WAVES; ++u) {
      const int t = wave + u * DR_WAVES;                 // instruction id: segment t / 16, row pair t % 16
      if (t < ns * 16) {                                 // uniform
        const int seg = t >> 4, ins = t & 15;
        const int r = ins * 2 + (lane >> 5);
        const int piece = min(ks0 * 2 + (s0 + seg) * 32 + ((lane & 31) ^ (r & 15)), last_piece);
        __builtin_amdgcn_global_load_lds(PARSE_DEC_GLB_PTR((const char *)a.x + (size_t)min(r, B - 1) * n * 2 + (size_t)piece * 16),
                                         PARSE_DEC_LDS_PTR(xs + seg * DR_SEG_BYTES + ins * 1024), 16, 0, 0);
      }
    }
  };
  // lane's x operand of step kl (counted from the first staged segment)
  auto x_operand = [&](int kl) -> u32x4 {
    return *reinterpret_cast<const u32x4 *>(xs + (kl >> 4) * DR_SEG_BYTES + j * 512 + ((((kl & 15) * 2 + q) ^ (j & 15)) * 16));
  };
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  const u32x4 zero = {0, 0, 0, 0};
  const char *vrow = (const char *)ly.Vt + ((size_t)rb * nkb + ks0) * 1024;   // uniform; operand k of the slice at + k KiB
  const int vlane = lane * 16;
  u32x4 vr[DR_MAXK];
  if (!TWO) {
    // ---- all Vt operands of this wavefront, requested at once (steps past the count re-read the last one) ----
#pragma unroll
    for (int g = 0; g < HK / 4; ++g) {                   // a slice of up to 128 steps: up to HK per wavefront
      if (g * 4 < cntAw) {                               // uniform
#pragma unroll
        for (int ii = 0; ii < 4; ++ii)
          vr[g * 4 + ii] = *reinterpret_cast<const u32x4 *>(vrow + (size_t)(a0 + min(g * 4 + ii, cntAw - 1)) * 1024 + vlane);
      } else {
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) vr[g * 4 + ii] = zero;
      }
    }
    stage_x(0, nsegA);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                     // everybody's x rows are in LDS
#pragma unroll
    for (int g = 0; g < HK / 4; ++g) {
      if (g * 4 < cntAw) {                               // uniform
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {
          const int i = g * 4 + ii;
          const u32x4 xv = x_operand(min(a0 + i, cntA - 1));
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(vr[i]), dec_bf16x8(i < cntAw ? xv : zero), acc, 0, 0, 0);
        }
      }
    }
  } else {
    // ---- Two stagings.  Here the x rows go through registers (16 loads of 1 KiB per wavefront and half, then 16 LDS
    // writes): with plain loads the compiler counts every outstanding load exactly, so the products of part A start while
    // the operands of part B are still in flight (it does not do that across loads that write LDS directly).  Every
    // wavefront issues the same number of loads whatever the counts are -- instructions past the end repeat the last
    // one (same data to the same place) -- first half of x, operands of part A, operands of part B ----
    constexpr int XI = DR_MAXSEG * 16 / DR_WAVES;        // x instructions per wavefront and half
    auto x_src = [&](int s0, int ns, int u) -> const char * {
      const int t = min(wave + u * DR_WAVES, ns * 16 - 1);
      const int seg = t >> 4, ins = t & 15;
      const int r = ins * 2 + (lane >> 5);
      const int piece = min(ks0 * 2 + (s0 + seg) * 32 + ((lane & 31) ^ (r & 15)), last_piece);
      return (const char *)a.x + (size_t)min(r, B - 1) * n * 2 + (size_t)piece * 16;
    };
    auto x_dst = [&](int ns, int u) -> char * {          // wave-uniform slot + the lane's 16 bytes
      const int t = min(wave + u * DR_WAVES, ns * 16 - 1);
      return xs + (t >> 4) * DR_SEG_BYTES + (t & 15) * 1024 + lane * 16;
    };
    auto bare_barrier = [&]() {     // the usual barrier comes with a fence that waits for every outstanding load
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    };
    u32x4 xr[XI];
#pragma unroll
    for (int u = 0; u < XI; ++u) xr[u] = *reinterpret_cast<const u32x4 *>(x_src(0, nsegA, u));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < HK; ++i)
      vr[i] = *reinterpret_cast<const u32x4 *>(vrow + (size_t)(a0 + min(i, max(cntAw - 1, 0))) * 1024 + vlane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < HK; ++i)
      vr[HK + i] = *reinterpret_cast<const u32x4 *>(vrow + (size_t)min(cntA + b0 + min(i, max(cntBw - 1, 0)), cnt_wg - 1) * 1024 + vlane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < XI; ++u) *reinterpret_cast<u32x4 *>(x_dst(nsegA, u)) = xr[u];
    bare_barrier();                                      // everybody's share of the first half of x is in LDS
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < HK; ++i) {
      const u32x4 xv = x_operand(min(a0 + i, cntA - 1));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(vr[i]), dec_bf16x8(i < cntAw ? xv : zero), acc, 0, 0, 0);
      if (i % 4 == 3) __builtin_amdgcn_sched_barrier(0);     // a few x operands in registers at a time, not all sixteen
    }
    bare_barrier();                                      // everybody is done with the first half of x
    __builtin_amdgcn_sched_barrier(0);
    const int nsegB = max(nseg - nsegA, 1);
#pragma unroll
    for (int u = 0; u < XI; ++u) xr[u] = *reinterpret_cast<const u32x4 *>(x_src(min(nsegA, nseg - 1), nsegB, u));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < XI; ++u) *reinterpret_cast<u32x4 *>(x_dst(nsegB, u)) = xr[u];
    bare_barrier();
    __builtin_amdgcn_sched_barrier(0);
    const int offB = cntA - nsegA * DR_SEG_KB;           // first step of part B counted from the first segment staged now (0)
#pragma unroll
    for (int i = 0; i < HK; ++i) {
      const u32x4 xv = x_operand(max(0, min(offB + b0 + i, offB + cntB - 1)));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(vr[HK + i]), dec_bf16x8(i < cntBw ? xv : zero), acc, 0, 0, 0);
      if (i % 4 == 3) __builtin_amdgcn_sched_barrier(0);
    }
  }
  __syncthreads();        // the staged rows are dead: their LDS now takes the wavefronts' sums
  float(*red)[16][64] = reinterpret_cast<float(*)[16][64]>(xs);               // [8][16][64] floats = 32 KiB
  float *sums = reinterpret_cast<float *>(xs + 32768);                        // [16][64]
#pragma unroll
  for (int e = 0; e < 16; ++e) red[wave][e][lane] = acc[e];
  __syncthreads();
  // the eight sums of each value, in wavefront order; value v = (e, lane)
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int v = (int)threadIdx.x + u * DR_THREADS;
    const float *r0 = &red[0][0][0] + v;
    float sum = r0[0];
#pragma unroll
    for (int w = 1; w < DR_WAVES; ++w) sum += r0[w * 1024];
    if (KS == 1) sums[v] = sum;
    else           // device-scope store: written through to memory, past this die's (non-coherent) L2
      __hip_atomic_store(&ly.zpart[((size_t)rb * KS + sl) * 1024 + v], sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (KS == 1) {
    __syncthreads();
    if (wave == 0) {
      float s[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = sums[e * 64 + lane];
      dec_store_z_operands(s, mask, lane, ly.zf, rb);
    }
    return;
  }
  // ---- ticket.  The partial sums and the ticket are device-scope accesses (they go past the die's L2, which is not
  // coherent with the other dies'), so no cache has to be written back or invalidated as a device-scope fence would do
  // (that would also throw away the x rows and factor lines the other workgroups of the die are using): every thread
  // waits until its own stores are acknowledged, the barrier collects all of them, then thread 0 draws ----
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const int t = __hip_atomic_fetch_add(&ly.ticket[rb], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = t == KS - 1 ? 1 : 0;
    if (last) __hip_atomic_store(&ly.ticket[rb], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
    am_last = last;
  }
  __syncthreads();
  if (!am_last) return;
  // the last workgroup of the block: all KS partial sums are in memory; read them past the L2 as well, add in slice order
  if (wave == 0) {
    float s[16];
    const float *zp = ly.zpart + (size_t)rb * KS * 1024 + lane;
#pragma unroll
    for (int e = 0; e < 16; ++e) s[e] = __hip_atomic_load(zp + e * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int o = 1; o < KS; ++o) {
      float t[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) t[e] = __hip_atomic_load(zp + (size_t)o * 1024 + e * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] += t[e];
    }
    dec_store_z_operands(s, mask, lane, ly.zf, rb);
  }
}

// ---------------------------------------------------------------------------------------------------------
// decode_zv: z for a handful of sequences (B <= 4), on the vector units.  With one to four sequences the 32-wide N side
// of the matrix instruction is almost empty and, worse, a 32-rank block per workgroup leaves most compute units without
// work (one sequence selects k groups: a 4096x4096 layer with 8 groups of 96 ranks has 24 blocks for 256 units).  Here a
// workgroup owns EIGHT ranks of a block over the whole reduction range: in the operand order the 16-byte pieces of 8
// consecutive ranks are 128 contiguous bytes, so a wavefront instruction reads 8 such lines (4 reduction steps x 2
// halves), every line exactly once in the launch.  Lane (step s of 4, half q, rank j of 8) multiplies its 8 factor values
// with the matching 8 values of each sequence's x row (all of x sits in LDS) and keeps one fp32 sum per sequence; the 8
// lanes of a rank are added by a butterfly, the eight wavefronts through LDS in wavefront order.  No partial sums leave
// the workgroup.  The result is masked, rounded and stored exactly like decode_zr's (one 16-byte piece per sequence).
constexpr int DV_WAVES = 8, DV_THREADS = DV_WAVES * 64;
constexpr int DV_JW = 8;                     // ranks per workgroup
constexpr int DV_DEPTH = 24;                 // factor loads a lane has in flight: reductions of up to 12288 in one batch
constexpr int DV_XBYTES = 96 * 1024;         // most LDS the x rows may take
constexpr int DV_MAXB = 4;

template <int NB>
__global__ __launch_bounds__(DV_THREADS) void decode_zv(DecArgs a) {
  int li = 0;
#pragma unroll
  for (int i = 1; i < DEC_MAX_LAYERS; ++i) li += (i < a.n_layers && (int)blockIdx.x >= a.L[i].z_first) ? 1 : 0;
  const DecLayer &ly = a.L[li];
  const int bid = blockIdx.x - ly.z_first;
  const int rb = bid / (32 / DV_JW), j0 = (bid % (32 / DV_JW)) * DV_JW;
  const int n = a.n, B = a.B;
  const uint32_t mask = (uint32_t)ly.plan[65 + (rb * 32) / ly.gs];
  if (mask == 0u) return;                    // a block nobody selected is neither read nor written
  extern __shared__ __attribute__((aligned(16))) char xs[];      // NB * n bf16: several workgroups fit a compute unit
  __shared__ float red[DV_WAVES][NB][DV_JW];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int jl = lane & 7, q = (lane >> 3) & 1, ks = lane >> 4;
  const int nkb = n / 16;
  const int ninstr = (nkb + 3) / 4;                                  // wavefront instructions of the block, 4 steps each
  const int nw = (ninstr - wave + DV_WAVES - 1) / DV_WAVES;          // ... of this wavefront: wave, wave + 4, ...
  const char *vbase = (const char *)ly.Vt + (size_t)rb * nkb * 1024 + (q * 32 + j0 + jl) * 16;
  u32x4 v[DV_DEPTH];
  auto request = [&](int i0) {               // lanes past the last step re-read it (switched off when used)
#pragma unroll
    for (int u = 0; u < DV_DEPTH; ++u) {
      if (i0 + u < nw) {                     // uniform
        const int kb = min(((wave + (i0 + u) * DV_WAVES) << 2) + ks, nkb - 1);
        v[u] = *reinterpret_cast<const u32x4 *>(vbase + (size_t)kb * 1024);
      }
    }
  };
  request(0);
  __builtin_amdgcn_sched_barrier(0);
  // the x rows: B * n contiguous bf16, copied as they are; rows B .. NB-1 (never stored) are cleared
  for (int i = threadIdx.x; i < NB * n / 8; i += DV_THREADS) {
    u32x4 w = {0, 0, 0, 0};
    if (i < B * n / 8) w = *reinterpret_cast<const u32x4 *>((const char *)a.x + (size_t)i * 16);
    *reinterpret_cast<u32x4 *>(xs + (size_t)i * 16) = w;
  }
  __syncthreads();
  float acc[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) acc[b] = 0.f;
  for (int i0 = 0; i0 < nw; i0 += DV_DEPTH) {
#pragma unroll
    for (int u = 0; u < DV_DEPTH; ++u) {
      if (i0 + u >= nw) break;               // uniform
      const int kbr = ((wave + (i0 + u) * DV_WAVES) << 2) + ks;
      const bool on = kbr < nkb;
      const int kb = min(kbr, nkb - 1);
      const u32x4 vv = v[u];
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const u32x4 xv = *reinterpret_cast<const u32x4 *>(xs + ((size_t)b * n + kb * 16 + q * 8) * 2);
        float t = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          t += __uint_as_float(vv[e] << 16) * __uint_as_float(xv[e] << 16);
          t += __uint_as_float(vv[e] & 0xFFFF0000u) * __uint_as_float(xv[e] & 0xFFFF0000u);
        }
        acc[b] += on ? t : 0.f;
      }
    }
    if (i0 + DV_DEPTH < nw) request(i0 + DV_DEPTH);     // uniform
  }
  // the 8 lanes of a rank (4 steps x 2 halves), then the wavefronts
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    float t = acc[b];
    t += __shfl_xor(t, 8, 64);
    t += __shfl_xor(t, 16, 64);
    t += __shfl_xor(t, 32, 64);
    if (lane < DV_JW) red[wave][b][lane] = t;
  }
  __syncthreads();
  if (threadIdx.x < 32) {                    // one 16-byte piece per sequence: its 8 ranks, zeros outside the group's mask
    const int b = threadIdx.x;
    u32x4 out = {0, 0, 0, 0};
    if (b < B && b < NB && ((mask >> b) & 1u)) {
      float s8[DV_JW];
#pragma unroll
      for (int e = 0; e < DV_JW; ++e) {
        float t = red[0][min(b, NB - 1)][e];
#pragma unroll
        for (int w = 1; w < DV_WAVES; ++w) t += red[w][min(b, NB - 1)][e];
        s8[e] = t;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) out[e] = cvt_pk_bf16(s8[2 * e], s8[2 * e + 1]);
    }
    *reinterpret_cast<u32x4 *>((char *)ly.zf + (size_t)(rb * 2 + (j0 >> 4)) * 1024 + (((j0 >> 3) & 1) * 32 + b) * 16) = out;
  }
}

// ---------------------------------------------------------------------------------------------------------
// decode_y: y.  grid = ceil(ncb / NC) workgroups per layer, each owns NC consecutive 32-column output blocks;
// wavefront w owns an eighth of the used reduction blocks for all NC column blocks, so one z operand (cache-resident)
// feeds NC products; the Ut operands of its first MAXK reduction blocks are requested at once (MAXK sized so that
// everything stays in registers), the rest is streamed in chunks; the eight wavefronts add up through LDS.
template <int NC>
__global__ __launch_bounds__(DY_THREADS) void decode_y(DecArgs a) {
  int li = 0;
#pragma unroll
  for (int i = 1; i < DEC_MAX_LAYERS; ++i) li += (i < a.n_layers && (int)blockIdx.x >= a.L[i].y_first) ? 1 : 0;
  const DecLayer &ly = a.L[li];
  const uint16_t *__restrict__ Ut = ly.Ut;
  const uint16_t *__restrict__ zf = ly.zf;
  const int32_t *__restrict__ plan = ly.plan;
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
  // count and ids come from the plan in one round trip (ids past the count are -1 and not used)
  const int n_used_raw = plan[0];
  if (threadIdx.x < DEC_MAXG) used[threadIdx.x] = plan[1 + threadIdx.x];
  const int n_used = max(0, min(n_used_raw, G));
  __syncthreads();
  const int kpg = gs / 16;                 // reduction blocks per group
  const int total_kb = n_used * kpg;       // selected reduction blocks
  for (int i = threadIdx.x; i < total_kb; i += DY_THREADS) kb_list[i] = max(used[i / kpg], 0) * kpg + i % kpg;
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

// ---------------------------------------------------------------------------------------------------------
// decode_yv: y for a handful of sequences (B <= 4), on the vector units -- the counterpart of decode_zv.  decode_y feeds
// z to the matrix cores as a 32-sequence operand (1 KiB per reduction block whatever B is) that every workgroup re-reads;
// here z is a few values per rank: a workgroup copies the B sequences' pieces of the used reduction blocks into LDS once
// (16 bytes per block half and sequence) and then streams nothing but Ut.  Workgroup = 8 * CG consecutive output columns
// of one layer (CG = 2 or 4 groups of 8 columns: 128-byte lines of the operand order, each read once in the launch);
// wavefront w owns column group w % CG and every (8 / CG)-th instruction of the used reduction blocks, 4 blocks per
// instruction: lane (block s of 4, half q, column j of 8) multiplies its 8 Ut values with the 8 matching z values of
// each sequence.  The 8 lanes of a column are added by a butterfly, the wavefronts of a column group through LDS in
// wavefront order; one 16-byte store per sequence and column group.
constexpr int DYV_WAVES = 8, DYV_THREADS = DYV_WAVES * 64;
constexpr int DYV_DEPTH = 16;                // Ut loads a lane has in flight
constexpr int DYV_ZBYTES = 96 * 1024;        // most LDS the z pieces may take

template <int NB, int CG>
__global__ __launch_bounds__(DYV_THREADS) void decode_yv(DecArgs a) {
  constexpr int PARTS = DYV_WAVES / CG;      // wavefronts that share a column group
  int li = 0;
#pragma unroll
  for (int i = 1; i < DEC_MAX_LAYERS; ++i) li += (i < a.n_layers && (int)blockIdx.x >= a.L[i].y_first) ? 1 : 0;
  const DecLayer &ly = a.L[li];
  const int32_t *__restrict__ plan = ly.plan;
  const int B = a.B, m = ly.m, G = ly.G, gs = ly.gs;
  const int bid = blockIdx.x - ly.y_first;
  extern __shared__ __attribute__((aligned(16))) char zs[];          // [used reduction block][half][NB] pieces of 16 bytes
  __shared__ int32_t kb_list[DY_MAXKB];
  __shared__ int32_t used[DEC_MAXG];
  __shared__ float red[DYV_WAVES][NB][8];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int jl = lane & 7, q = (lane >> 3) & 1, ks = lane >> 4;
  const int cg = wave % CG, part = wave / CG;
  const int ncb = m / 32;
  const int col0 = (bid * CG + cg) * 8;                              // first column of this wavefront's group
  const int n_used_raw = plan[0];
  if (threadIdx.x < DEC_MAXG) used[threadIdx.x] = plan[1 + threadIdx.x];
  const int n_used = max(0, min(n_used_raw, G));
  __syncthreads();
  const int kpg = gs / 16;
  const int total_kb = n_used * kpg;
  for (int i = threadIdx.x; i < total_kb; i += DYV_THREADS) kb_list[i] = max(used[i / kpg], 0) * kpg + i % kpg;
  __syncthreads();
  // z pieces of the used blocks: piece (i, h, b) = ranks kb_list[i]*16 + 8h .. +7 of sequence b (zeros for b >= B)
  for (int t = threadIdx.x; t < total_kb * 2 * NB; t += DYV_THREADS) {
    const int b = t % NB, h = (t / NB) & 1, i = t / (2 * NB);
    u32x4 w = {0, 0, 0, 0};
    if (b < B) w = *reinterpret_cast<const u32x4 *>((const char *)ly.zf + (size_t)kb_list[i] * 1024 + (h * 32 + b) * 16);
    *reinterpret_cast<u32x4 *>(zs + (size_t)t * 16) = w;
  }
  const int ninstr = (total_kb + 3) / 4;
  const int nw = col0 < m ? (ninstr - part + PARTS - 1) / PARTS : 0;  // instructions of this wavefront: part, part + PARTS, ...
  // column col0 + jl sits in column block c / 32 at place c % 32 of the operand
  const int cc = min(col0, m - 8) + jl;
  const char *ubase = (const char *)ly.Ut + (size_t)(cc >> 5) * 1024 + (q * 32 + (cc & 31)) * 16;
  const size_t ustep = (size_t)ncb * 1024;
  u32x4 v[DYV_DEPTH];
  auto request = [&](int i0) {               // lanes past the last block re-read it (switched off when used)
#pragma unroll
    for (int u = 0; u < DYV_DEPTH; ++u) {
      if (i0 + u < nw) {                     // uniform
        const int i = min(((part + (i0 + u) * PARTS) << 2) + ks, total_kb - 1);
        v[u] = *reinterpret_cast<const u32x4 *>(ubase + (size_t)kb_list[i] * ustep);
      }
    }
  };
  request(0);
  __syncthreads();                           // the z pieces are in LDS
  float acc[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) acc[b] = 0.f;
  for (int i0 = 0; i0 < nw; i0 += DYV_DEPTH) {
#pragma unroll
    for (int u = 0; u < DYV_DEPTH; ++u) {
      if (i0 + u >= nw) break;               // uniform
      const int ir = ((part + (i0 + u) * PARTS) << 2) + ks;
      const bool on = ir < total_kb;
      const int i = min(ir, total_kb - 1);
      const u32x4 uv = v[u];
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const u32x4 zv = *reinterpret_cast<const u32x4 *>(zs + (size_t)((i * 2 + q) * NB + b) * 16);
        float t = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          t += __uint_as_float(uv[e] << 16) * __uint_as_float(zv[e] << 16);
          t += __uint_as_float(uv[e] & 0xFFFF0000u) * __uint_as_float(zv[e] & 0xFFFF0000u);
        }
        acc[b] += on ? t : 0.f;
      }
    }
    if (i0 + DYV_DEPTH < nw) request(i0 + DYV_DEPTH);   // uniform
  }
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    float t = acc[b];
    t += __shfl_xor(t, 8, 64);
    t += __shfl_xor(t, 16, 64);
    t += __shfl_xor(t, 32, 64);
    if (lane < 8) red[wave][b][lane] = t;
  }
  __syncthreads();
  if ((int)threadIdx.x < CG * NB) {          // thread (column group, sequence): 8 columns = one 16-byte store
    const int g2 = threadIdx.x / NB, b = threadIdx.x % NB;
    const int c = (bid * CG + g2) * 8;
    if (b < B && c < m) {
      u32x4 out;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int pt = 0; pt < PARTS; ++pt) { s0 += red[pt * CG + g2][b][2 * e]; s1 += red[pt * CG + g2][b][2 * e + 1]; }
        out[e] = pack_bf16x2(s0, s1);
      }
      *reinterpret_cast<u32x4 *>(ly.y + (size_t)b * m + c) = out;
    }
  }
}

// workspace of one layer: z in operand order (R/16 operands of 1 KiB), then the partial sums of decode_zr
static size_t dec_zf_bytes(const parse_layer *L) { return round_up((size_t)(L->R / 16) * 1024, 256); }
// decode_zr takes reductions of up to DR_MAX_KS slices of 8 * DR_MAXK steps (n <= 65536) and layers of up to DEC_TICKETS
// rank blocks whose groups are whole 32-rank blocks (which the operand-order layout requires anyway)
static bool dec_zr_ok(const parse_layer *L) {
  if (L->G <= 0 || L->R % L->G != 0 || (L->R / L->G) % 32 != 0) return false;
  if (L->R / 32 > DEC_TICKETS) return false;
  const int nkb = L->n / 16;
  return (nkb + 8 * DR_MAXK - 1) / (8 * DR_MAXK) <= DR_MAX_KS;
}
// slices of the reduction range: enough that a slice fits a workgroup (8 * DR_MAXK steps), and enough workgroups to give
// every compute unit one
static int dec_zr_slices(const parse_layer *layers, int n_layers) {
  const int nkb = layers[0].n / 16;
  int blocks = 0;
  for (int l = 0; l < n_layers; ++l) blocks += layers[l].R / 32;
  const int need = (nkb + 8 * DR_MAXK - 1) / (8 * DR_MAXK);
  int ks = blocks > 0 ? DR_TARGET_WGS / blocks : 1;
  if (ks > nkb / 8) ks = nkb / 8;          // at least one step per wavefront
  if (ks < need) ks = need;
  if (ks > DR_MAX_KS) ks = DR_MAX_KS;
  return ks < 1 ? 1 : ks;
}
static size_t dec_zpart_bytes(const parse_layer *L, int ks) { return ks > 1 ? (size_t)(L->R / 32) * ks * 4096 : 0; }
size_t decode_plan_bytes(int n_layers) { return round_up((size_t)n_layers * DEC_PLAN_WORDS * sizeof(int32_t), 256); }
// z workspace of several layers that go through one call: per layer z, then its partial sums
size_t decode_z_bytes(const parse_layer *layers, int n_layers) {
  const int ks = dec_zr_slices(layers, n_layers);
  size_t t = 0;
  for (int l = 0; l < n_layers; ++l) t += dec_zf_bytes(&layers[l]) + dec_zpart_bytes(&layers[l], ks);
  return t;
}
// one layer's intermediates, then room for a one-layer plan (used when the caller brings no plan)
size_t decode_workspace_bytes(const parse_layer *L) { return decode_z_bytes(L, 1) + decode_plan_bytes(1); }

bool decode_supported(const parse_layer *L) {
  return L->R / 16 <= DY_MAXKB && L->G <= DEC_MAXG && L->n % 16 == 0 && L->n >= 16 && dec_zr_ok(L);
}

int build_decode_plan(const parse_layer *layers, const parse_patterns *pts, int n_layers, const int32_t *pattern_id,
                      int B, int32_t *plan, hipStream_t s) {
  if (n_layers < 1 || n_layers > DEC_MAX_LAYERS) return PARSE_ESHAPE;
  DecPlanArgs pa{};
  for (int l = 0; l < n_layers; ++l) {
    pa.subsets[l] = pts[l].subsets; pa.stride[l] = pts[l].subset_stride; pa.k[l] = pts[l].k;
    pa.n_patterns[l] = pts[l].n_patterns; pa.G[l] = layers[l].G;
  }
  pa.pattern_id = pattern_id; pa.B = B; pa.plan = plan;
  hipLaunchKernelGGL(decode_plan_build, dim3(n_layers), dim3(64), 0, s, pa);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

// n_layers layers that share x (same n); plan = n_layers consecutive layer plans; Y[l] and the z part of layer l in the
// workspace follow the order of `layers`.
int forward_decode_planned_bf16(const parse_layer *layers, int n_layers, const uint16_t *x, int B, int32_t *plan,
                                uint16_t *const *Y, void *workspace, hipStream_t s) {
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
  a.B = B;
  a.n = layers[0].n;
  for (int l = 0; l < n_layers; ++l) {
    if (!decode_supported(&layers[l])) return PARSE_ESHAPE;
    if (layers[l].n != a.n) return PARSE_ESHAPE;
  }
  // column blocks per workgroup (one z operand feeds NC products): the smallest count that puts at most one
  // workgroup on a compute unit -- a unit with two streams runs both at half the rate and sets the kernel's time
  int NC = 1;
  for (; NC < 4; ++NC) {
    int wgs = 0;
    for (int l = 0; l < n_layers; ++l) wgs += (layers[l].m / 32 + NC - 1) / NC;
    if (wgs <= n_cu) break;
  }
  const int KS = dec_zr_slices(layers, n_layers);
  a.KS = KS;
  char *ws = reinterpret_cast<char *>(workspace);
  int zb = 0, yb = 0;
  for (int l = 0; l < n_layers; ++l) {
    const parse_layer *L = &layers[l];
    DecLayer &d = a.L[l];
    d.Vt = (const uint16_t *)L->Vt;
    d.Ut = (const uint16_t *)L->Ut;
    d.y = Y[l];
    d.zf = reinterpret_cast<uint16_t *>(ws);
    ws += dec_zf_bytes(L);
    d.zpart = reinterpret_cast<float *>(ws);
    ws += dec_zpart_bytes(L, KS);
    d.plan = plan + (size_t)l * DEC_PLAN_WORDS;
    d.ticket = plan + (size_t)l * DEC_PLAN_WORDS + 192;
    d.R = L->R; d.G = L->G; d.gs = L->R / L->G; d.m = L->m;
    d.z_first = zb; zb += (L->R / 32) * KS;
    d.y_first = yb; yb += (L->m / 32 + NC - 1) / NC;
  }
  const int nkb = a.n / 16;
  const int NB = B <= 1 ? 1 : (B <= 2 ? 2 : 4);
  if (B <= DV_MAXB && (size_t)NB * a.n * 2 <= (size_t)DV_XBYTES) {
    // a handful of sequences: eight ranks per workgroup on the vector units, no split of the reduction range
    zb = 0;
    for (int l = 0; l < n_layers; ++l) { a.L[l].z_first = zb; zb += (layers[l].R / 32) * (32 / DV_JW); }
    const size_t lds = (size_t)NB * a.n * 2;
    if (NB == 1) {
      PARSE_ALLOW_LDS(decode_zv<1>, lds);
      hipLaunchKernelGGL(decode_zv<1>, dim3(zb), dim3(DV_THREADS), lds, s, a);
    } else if (NB == 2) {
      PARSE_ALLOW_LDS(decode_zv<2>, lds);
      hipLaunchKernelGGL(decode_zv<2>, dim3(zb), dim3(DV_THREADS), lds, s, a);
    } else {
      PARSE_ALLOW_LDS(decode_zv<4>, lds);
      hipLaunchKernelGGL(decode_zv<4>, dim3(zb), dim3(DV_THREADS), lds, s, a);
    }
  } else {
    const bool two = (nkb + KS - 1) / KS > DR_HALF_KB;     // the longest slice needs two stagings of x
    if (two) hipLaunchKernelGGL(decode_zr<true>, dim3(zb), dim3(DR_THREADS), 0, s, a);
    else hipLaunchKernelGGL(decode_zr<false>, dim3(zb), dim3(DR_THREADS), 0, s, a);
  }
  PARSE_LAUNCH_CHECK();
  size_t max_kb = 0;
  for (int l = 0; l < n_layers; ++l) max_kb = std::max(max_kb, (size_t)layers[l].R / 16);
  const size_t zs_bytes = max_kb * 2 * NB * 16;            // z pieces of every reduction block a layer has
  if (B <= DV_MAXB && zs_bytes <= (size_t)DYV_ZBYTES) {
    // a handful of sequences: z as a few values per rank in LDS, the launch streams only Ut.  16 columns per workgroup
    // unless that makes more than about four workgroups per compute unit
    int cols = 0;
    for (int l = 0; l < n_layers; ++l) cols += layers[l].m;
    const int CG = cols / 16 > 4 * n_cu ? 4 : 2;
    yb = 0;
    for (int l = 0; l < n_layers; ++l) { a.L[l].y_first = yb; yb += (layers[l].m + 8 * CG - 1) / (8 * CG); }
#define PARSE_YV(NB_, CG_)                                                                     \
  do {                                                                                         \
    PARSE_ALLOW_LDS((decode_yv<NB_, CG_>), zs_bytes);                                          \
    hipLaunchKernelGGL((decode_yv<NB_, CG_>), dim3(yb), dim3(DYV_THREADS), zs_bytes, s, a);    \
  } while (0)
    if (NB == 1) { if (CG == 2) PARSE_YV(1, 2); else PARSE_YV(1, 4); }
    else if (NB == 2) { if (CG == 2) PARSE_YV(2, 2); else PARSE_YV(2, 4); }
    else { if (CG == 2) PARSE_YV(4, 2); else PARSE_YV(4, 4); }
#undef PARSE_YV
  } else if (NC == 1) hipLaunchKernelGGL(decode_y<1>, dim3(yb), dim3(DY_THREADS), 0, s, a);
  else if (NC == 2) hipLaunchKernelGGL(decode_y<2>, dim3(yb), dim3(DY_THREADS), 0, s, a);
  else if (NC == 3) hipLaunchKernelGGL(decode_y<3>, dim3(yb), dim3(DY_THREADS), 0, s, a);
  else hipLaunchKernelGGL(decode_y<4>, dim3(yb), dim3(DY_THREADS), 0, s, a);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

// Without a caller's plan: the plan is built into the workspace (after the z parts), one more small launch.
int forward_decode_multi_bf16(const parse_layer *layers, const parse_patterns *pts, int n_layers, const uint16_t *x,
                              int B, const int32_t *pattern_id, uint16_t *const *Y, void *workspace, hipStream_t s) {
  if (n_layers < 1 || n_layers > DEC_MAX_LAYERS) return PARSE_ESHAPE;
  int32_t *plan = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(workspace) + decode_z_bytes(layers, n_layers));
  int st = build_decode_plan(layers, pts, n_layers, pattern_id, B, plan, s);
  if (st != PARSE_OK) return st;
  return forward_decode_planned_bf16(layers, n_layers, x, B, plan, Y, workspace, s);
}

int forward_decode_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *x, int B,
                        const int32_t *pattern_id, uint16_t *y, void *workspace, hipStream_t s) {
  uint16_t *Y[1] = {y};
  return forward_decode_multi_bf16(L, pt, 1, x, B, pattern_id, Y, workspace, s);
}

}  // namespace parse
