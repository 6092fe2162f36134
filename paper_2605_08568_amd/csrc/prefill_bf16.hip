// a6: fused prefill kernel for bf16 PARSE_MFMA16 layers:  Y = (X Vt_S^T) Ut_S  (Sec. 4.4, Eq. 10) with the
// r_S-wide intermediate Z kept on chip.
//
// One workgroup (4 wavefronts) owns BM consecutive token rows and the whole active rank r_S:
//   phase 1  Z^T tiles = Vt_S-operand x X-tile on the bf16 matrix cores (32x32x16, fp32 accumulate).  The
//            factor operands come straight from global memory in operand order (one coalesced 1 KiB
//            fetch per wavefront instruction, no LDS hop); the X tile is staged in LDS because all four
//            wavefronts share it.  The accumulators are rounded to bf16 and written to the Z block in LDS.
//   phase 2  Y^T tiles = Ut_S-operand x Z (read from LDS), stored as bf16.
// Both products are computed transposed (factor = A operand with M = ranks / output columns, tokens = N)
// so that the accumulator layout gives each lane 4 consecutive ranks (phase 1: one 8-byte LDS store) and
// 4 consecutive output columns (phase 2: one 8-byte global store).
// A BM-row block of the flat token axis that spans several prompts is processed once per prompt segment.
//
// The inner loops are branch-free: the number of 32-wide operand blocks a wavefront owns in a pass (NB) is a
// template parameter, prefetches past the end are clamped to the last valid operand instead of being
// predicated, and shapes that do not fill whole staged tiles take a separate, simpler kernel.
#include "prefill_common.hpp"

namespace parse {

// ---------------------------------------------------------------------------------------------------------
// phase 1, one pass: this wavefront's NB rank blocks (first one rb0, then every 4th) x all BM tokens.
// Requires n % (2*PF_BK) == 0.
template <int BM, int NB>
__device__ __forceinline__ void phase1_pass(const PfArgs &a, const uint16_t *Vp, int row0, int rb0, uint16_t *Zs,
                                            int zld, uint16_t *Xs) {
  constexpr int NT = BM / 32;
  constexpr int XP = BM * PF_BK / 8 / PF_THREADS;
  constexpr int xld = PF_BK + PF_XPAD;
  const int lane = threadIdx.x & 63, l32 = lane & 31, q = lane >> 5;
  const int n = a.n, nkb = n / 16, nkt = n / PF_BK;
  f32x16 acc[NT][NB];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][i][e] = 0.f;
  const uint16_t *vbase[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) vbase[i] = Vp + ((size_t)(rb0 + 4 * i) * nkb * 64 + lane) * 8;
  // X tile pieces of this lane: piece = i*256 + tid -> row piece/8, column (piece%8)*8
  const uint16_t *xsrc[XP];
  int xdst[XP];
#pragma unroll
  for (int i = 0; i < XP; ++i) {
    const int piece = i * PF_THREADS + threadIdx.x;
    const int r = piece / (PF_BK / 8), c = (piece % (PF_BK / 8)) * 8;
    xsrc[i] = a.X + (size_t)min(row0 + r, a.rows - 1) * n + c;
    xdst[i] = r * xld + c;
  }
  const int xoff = l32 * xld + q * 8;   // operand read: token l32 (+32 t), reduction offset 16 s + 8 q
  u32x4 xr[2][XP];
  u32x4 vr[PF_DEPTH][NB];
  __syncthreads();  // earlier readers of Xs / Zs are done
#pragma unroll
  for (int i = 0; i < XP; ++i) xr[0][i] = *reinterpret_cast<const u32x4 *>(xsrc[i]);
#pragma unroll
  for (int d = 0; d < PF_DEPTH; ++d)
#pragma unroll
    for (int i = 0; i < NB; ++i) vr[d][i] = *reinterpret_cast<const u32x4 *>(vbase[i] + (size_t)d * 512);
#pragma unroll
  for (int i = 0; i < XP; ++i) xr[1][i] = *reinterpret_cast<const u32x4 *>(xsrc[i] + PF_BK);
#pragma unroll
  for (int i = 0; i < XP; ++i) *reinterpret_cast<u32x4 *>(Xs + xdst[i]) = xr[0][i];
  __syncthreads();
  for (int kt0 = 0; kt0 < nkt; kt0 += 2) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int kt = kt0 + u;   // LDS buffer = u (kt0 is even)
      // tile kt+2 replaces tile kt in the register ring (tile kt went to LDS one iteration ago)
      const int ktn = min(kt + 2, nkt - 1);
#pragma unroll
      for (int i = 0; i < XP; ++i) xr[u][i] = *reinterpret_cast<const u32x4 *>(xsrc[i] + (size_t)ktn * PF_BK);
      bf16x8 xb[2][NT];
#pragma unroll
      for (int t = 0; t < NT; ++t)
        xb[0][t] = as_bf16x8(*reinterpret_cast<const u32x4 *>(Xs + u * BM * xld + t * 32 * xld + xoff));
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (s < 3) {
#pragma unroll
          for (int t = 0; t < NT; ++t)
            xb[(s + 1) & 1][t] =
                as_bf16x8(*reinterpret_cast<const u32x4 *>(Xs + u * BM * xld + t * 32 * xld + xoff + (s + 1) * 16));
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the next step's LDS reads ahead of this step's matrix work
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
          for (int t = 0; t < NT; ++t)
            acc[t][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vr[u * 4 + s][i]), xb[s & 1][t], acc[t][i], 0, 0, 0);
        // the slot just consumed is refilled with the operands PF_DEPTH steps ahead
        const int kbn = min(kt * 4 + s + PF_DEPTH, nkb - 1);
#pragma unroll
        for (int i = 0; i < NB; ++i) vr[u * 4 + s][i] = *reinterpret_cast<const u32x4 *>(vbase[i] + (size_t)kbn * 512);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < XP; ++i) *reinterpret_cast<u32x4 *>(Xs + (u ^ 1) * BM * xld + xdst[i]) = xr[u ^ 1][i];
      __syncthreads();
    }
  }
  // accumulators -> bf16 -> Z block.  lane holds token l32 of block t, ranks rb*32 + 8*blk + 4*q + (0..3)
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        u32x2 w;
        w[0] = cvt_pk_bf16(acc[t][i][blk * 4 + 0], acc[t][i][blk * 4 + 1]);
        w[1] = cvt_pk_bf16(acc[t][i][blk * 4 + 2], acc[t][i][blk * 4 + 3]);
        *reinterpret_cast<u32x2 *>(Zs + (size_t)(t * 32 + l32) * zld + (rb0 + 4 * i) * 32 + blk * 8 + q * 4) = w;
      }
}

// phase 2, one pass: NB consecutive 32-column blocks starting at cb0 x all BM tokens; reduction over r_S.
// Requires rS % (16*PF_DEPTH) == 0.
template <int BM, int NB>
__device__ __forceinline__ void phase2_pass(const PfArgs &a, const uint16_t *Up, bool valid, int row0, int seg_lo,
                                            int seg_hi, int cb0, const uint16_t *Zs, int zld) {
  constexpr int NT = BM / 32;
  const int lane = threadIdx.x & 63, l32 = lane & 31, q = lane >> 5;
  const int m = a.m, ncb = m / 32, nk2 = a.rS / 16;
  f32x16 acc[NT][NB];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][i][e] = 0.f;
  const uint16_t *ubase = Up + ((size_t)cb0 * 64 + lane) * 8;   // + kb * ncb * 512 + i * 512
  const size_t kstride = (size_t)ncb * 512;
  const int zoff = l32 * zld + q * 8;
  u32x4 ua[PF_DEPTH][NB];
#pragma unroll
  for (int d = 0; d < PF_DEPTH; ++d)
#pragma unroll
    for (int i = 0; i < NB; ++i) ua[d][i] = *reinterpret_cast<const u32x4 *>(ubase + d * kstride + i * 512);
  bf16x8 zb[2][NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) zb[0][t] = as_bf16x8(*reinterpret_cast<const u32x4 *>(Zs + t * 32 * zld + zoff));
  for (int kb0 = 0; kb0 < nk2; kb0 += PF_DEPTH) {
#pragma unroll
    for (int d = 0; d < PF_DEPTH; ++d) {
      const int kb = kb0 + d;
      const int kbz = min(kb + 1, nk2 - 1);
#pragma unroll
      for (int t = 0; t < NT; ++t)
        zb[(d + 1) & 1][t] = as_bf16x8(*reinterpret_cast<const u32x4 *>(Zs + t * 32 * zld + zoff + kbz * 16));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[t][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ua[d][i]), zb[d & 1][t], acc[t][i], 0, 0, 0);
      const int kbn = min(kb + PF_DEPTH, nk2 - 1);
#pragma unroll
      for (int i = 0; i < NB; ++i) ua[d][i] = *reinterpret_cast<const u32x4 *>(ubase + kbn * kstride + i * 512);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // store: lane holds token t*32 + l32, columns (cb0+i)*32 + 8*blk + 4*q + (0..3)
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int r = row0 + t * 32 + l32;
    if (r < seg_lo || r >= seg_hi) continue;
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        u32x2 w;
        w[0] = valid ? cvt_pk_bf16(acc[t][i][blk * 4 + 0], acc[t][i][blk * 4 + 1]) : 0u;
        w[1] = valid ? cvt_pk_bf16(acc[t][i][blk * 4 + 2], acc[t][i][blk * 4 + 3]) : 0u;
        *reinterpret_cast<u32x2 *>(a.Y + (size_t)r * m + (cb0 + i) * 32 + blk * 8 + q * 4) = w;
      }
  }
}

template <int BM>
__global__ __launch_bounds__(PF_THREADS) void prefill_fused(PfArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const int zld = a.rS + PF_ZPAD;
  constexpr int xld = PF_BK + PF_XPAD;
  uint16_t *Zs = lds;                          // [BM][zld]
  uint16_t *Xs = lds + (size_t)BM * zld;       // [2][BM][xld]
  const int wave = threadIdx.x >> 6;
  const int row0 = xcd_tile(blockIdx.x, gridDim.x) * BM;
  const int row_end = min(row0 + BM, a.rows);
  const int nrb = a.rS / 32, ncb = a.m / 32;
  int seg_lo = row0;
  while (seg_lo < row_end) {
    const int p = prompt_of_row(a.tok_offsets, a.P, seg_lo);
    int seg_hi = (p + 1 < a.P) ? a.tok_offsets[p + 1] : a.rows;
    seg_hi = min(max(seg_hi, seg_lo + 1), row_end);
    const int pid = a.pattern_id[p];
    const bool valid = pid >= 0 && pid < a.n_patterns;
    const uint16_t *Vp = a.Vt_S + (valid ? (size_t)pid * a.rS * a.n : 0);
    const uint16_t *Up = a.Ut_S + (valid ? (size_t)pid * a.rS * a.m : 0);

    // phase 1: wave w owns rank blocks w, w+4, ...; a pass takes up to 4 of them (all waves run every pass:
    // the staged X tile is shared and the barriers are collective; a wave with nothing left recomputes its
    // last block, which rewrites the same Z values)
    const int my_nrb = max(1, (nrb - wave + 3) / 4);
    const int passes1 = (nrb + 15) / 16;
    for (int pass = 0; pass < passes1; ++pass) {
      int first = pass * 4;                       // index into this wave's own list of rank blocks
      int nb = min(4, my_nrb - first);
      if (nb <= 0) { first = my_nrb - 1; nb = 1; }
      const int rb0 = min(first * 4 + wave, nrb - 1);
      switch (nb) {
        case 4: phase1_pass<BM, 4>(a, Vp, row0, rb0, Zs, zld, Xs); break;
        case 3: phase1_pass<BM, 3>(a, Vp, row0, rb0, Zs, zld, Xs); break;
        case 2: phase1_pass<BM, 2>(a, Vp, row0, rb0, Zs, zld, Xs); break;
        default: phase1_pass<BM, 1>(a, Vp, row0, rb0, Zs, zld, Xs); break;
      }
    }
    __syncthreads();  // Z block complete

    // phase 2: a pass covers 16 column blocks, 4 consecutive ones per wave
    const int passes2 = (ncb + 15) / 16;
    for (int pass = 0; pass < passes2; ++pass) {
      const int cb0 = pass * 16 + wave * 4;
      const int nb = min(4, ncb - cb0);
      switch (nb) {
        case 4: phase2_pass<BM, 4>(a, Up, valid, row0, seg_lo, seg_hi, cb0, Zs, zld); break;
        case 3: phase2_pass<BM, 3>(a, Up, valid, row0, seg_lo, seg_hi, cb0, Zs, zld); break;
        case 2: phase2_pass<BM, 2>(a, Up, valid, row0, seg_lo, seg_hi, cb0, Zs, zld); break;
        case 1: phase2_pass<BM, 1>(a, Up, valid, row0, seg_lo, seg_hi, cb0, Zs, zld); break;
        default: break;
      }
    }
    seg_lo = seg_hi;
  }
}

// ---------------------------------------------------------------------------------------------------------
// Any shape the operand order allows (n % 16 == 0, r_S % 32 == 0, m % 32 == 0): same data flow, one matrix
// instruction deep, predicated.  Used when n is not a multiple of 128 or r_S not a multiple of 128.
template <int BM>
__global__ __launch_bounds__(PF_THREADS) void prefill_fused_any(PfArgs a) {
  constexpr int NT = BM / 32;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const int zld = a.rS + PF_ZPAD;
  constexpr int xld = PF_BK + PF_XPAD;
  uint16_t *Zs = lds;
  uint16_t *Xs = lds + (size_t)BM * zld;       // one buffer is enough here
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, q = lane >> 5;
  const int n = a.n, m = a.m, rS = a.rS;
  const int row0 = xcd_tile(blockIdx.x, gridDim.x) * BM;
  const int row_end = min(row0 + BM, a.rows);
  const int nkb = n / 16, nrb = rS / 32, ncb = m / 32, nk2 = rS / 16;
  int seg_lo = row0;
  while (seg_lo < row_end) {
    const int p = prompt_of_row(a.tok_offsets, a.P, seg_lo);
    int seg_hi = (p + 1 < a.P) ? a.tok_offsets[p + 1] : a.rows;
    seg_hi = min(max(seg_hi, seg_lo + 1), row_end);
    const int pid = a.pattern_id[p];
    const bool valid = pid >= 0 && pid < a.n_patterns;
    const uint16_t *Vp = a.Vt_S + (valid ? (size_t)pid * rS * n : 0);
    const uint16_t *Up = a.Ut_S + (valid ? (size_t)pid * rS * m : 0);
    // phase 1: a round handles rank blocks rbase + wave
    for (int rbase = 0; rbase < nrb; rbase += 4) {
      const int rb = min(rbase + wave, nrb - 1);
      f32x16 acc[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
      for (int k0 = 0; k0 < n; k0 += PF_BK) {
        __syncthreads();
        for (int piece = threadIdx.x; piece < BM * PF_BK / 8; piece += PF_THREADS) {
          const int r = piece / (PF_BK / 8), c = (piece % (PF_BK / 8)) * 8;
          const int gr = min(row0 + r, a.rows - 1), gc = k0 + c;
          const u32x4 v = (gc < n) ? *reinterpret_cast<const u32x4 *>(a.X + (size_t)gr * n + gc) : u32x4{0, 0, 0, 0};
          *reinterpret_cast<u32x4 *>(Xs + r * xld + c) = v;
        }
        __syncthreads();
        const int steps = min(4, (n - k0) / 16);
        for (int s = 0; s < steps; ++s) {
          const int kb = k0 / 16 + s;
          const bf16x8 va = as_bf16x8(*reinterpret_cast<const u32x4 *>(Vp + (((size_t)rb * nkb + kb) * 64 + lane) * 8));
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const bf16x8 xb = as_bf16x8(*reinterpret_cast<const u32x4 *>(Xs + (t * 32 + l32) * xld + s * 16 + q * 8));
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, xb, acc[t], 0, 0, 0);
          }
        }
      }
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
          u32x2 w;
          w[0] = cvt_pk_bf16(acc[t][blk * 4 + 0], acc[t][blk * 4 + 1]);
          w[1] = cvt_pk_bf16(acc[t][blk * 4 + 2], acc[t][blk * 4 + 3]);
          *reinterpret_cast<u32x2 *>(Zs + (size_t)(t * 32 + l32) * zld + rb * 32 + blk * 8 + q * 4) = w;
        }
    }
    __syncthreads();
    // phase 2
    for (int cb = wave; cb < ncb; cb += 4) {
      f32x16 acc[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
      for (int kb = 0; kb < nk2; ++kb) {
        const bf16x8 ua = as_bf16x8(*reinterpret_cast<const u32x4 *>(Up + (((size_t)kb * ncb + cb) * 64 + lane) * 8));
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const bf16x8 zb = as_bf16x8(*reinterpret_cast<const u32x4 *>(Zs + (size_t)(t * 32 + l32) * zld + kb * 16 + q * 8));
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua, zb, acc[t], 0, 0, 0);
        }
      }
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int r = row0 + t * 32 + l32;
        if (r < seg_lo || r >= seg_hi) continue;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
          u32x2 w;
          w[0] = valid ? cvt_pk_bf16(acc[t][blk * 4 + 0], acc[t][blk * 4 + 1]) : 0u;
          w[1] = valid ? cvt_pk_bf16(acc[t][blk * 4 + 2], acc[t][blk * 4 + 3]) : 0u;
          *reinterpret_cast<u32x2 *>(a.Y + (size_t)r * m + cb * 32 + blk * 8 + q * 4) = w;
        }
      }
    }
    __syncthreads();   // Zs is rewritten by the next segment
    seg_lo = seg_hi;
  }
}

size_t prefill_lds_bytes(int BM, int rS) {
  return ((size_t)BM * (rS + PF_ZPAD) + 2 * (size_t)BM * (PF_BK + PF_XPAD)) * sizeof(uint16_t);
}

constexpr size_t kLdsLimit = 160 * 1024;

template <typename K>
static int launch_prefill(K kernel, bool *attr_done, const PfArgs &a, int BM, size_t lds, hipStream_t s) {
  if (!*attr_done) {
    PARSE_HIP_TRY(hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit));
    *attr_done = true;
  }
  hipLaunchKernelGGL(kernel, dim3((a.rows + BM - 1) / BM), dim3(PF_THREADS), lds, s, a);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

// two-launch form (prefill_split_bf16.hip)
size_t prefill_split_workspace_bytes(int rows, int rS);
bool prefill_split_supported(int n, int rS);
int forward_prefill_split_bf16(const PfArgs &p, uint16_t *Z, int avg_prompt_rows, hipStream_t s);

// planned form (plan.hip, prefill_lds_bf16.hip)
size_t prefill_plan_bytes(int rows, int P, int n_patterns);
int prefill_plan_capacity(int rows, int P, int n_patterns);
bool prefill_plan_supported(int P, int n_patterns);
int build_prefill_plan(const int32_t *tok_offsets, const int32_t *pattern_id, int P, int rows, int n_patterns,
                       int32_t *plan, hipStream_t s);
size_t prefill_planned_z_bytes(int cap_tiles, int rS, int ks);
int prefill_planned_split(int rows, int n);
bool prefill_planned_supported(int n, int m, int rS);
int forward_prefill_planned_bf16(const PfArgs &p, const int32_t *plan, int cap, uint16_t *Z, int avg_prompt_rows,
                                 hipStream_t s);

int forward_prefill_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *X, int rows,
                         const int32_t *tok_offsets, const int32_t *pattern_id, int P, uint16_t *Y, void *workspace,
                         size_t workspace_bytes, hipStream_t s) {
  const int gs = L->R / L->G, rS = pt->k * gs;
  PfArgs a{X, (const uint16_t *)pt->Vt_S, (const uint16_t *)pt->Ut_S, Y, tok_offsets, pattern_id,
           pt->n_patterns, rows, L->n, L->m, rS, P};
  if (pt->n_shared > 0) {   // shared head: operands from two blocks (planned and two-launch schedules; the fused kernel has none)
    a.Vt_sh = (const uint16_t *)pt->Vt_shared;
    a.Ut_sh = (const uint16_t *)pt->Ut_shared;
    a.sh_ranks = pt->n_shared * gs;
  }
  const int schedule = pt->schedule;
  if (schedule < PARSE_SCHED_AUTO || schedule > PARSE_SCHED_PLANNED) return PARSE_EINVAL;
  // planned: plan + two launches of the LDS-staged tile kernel; workspace = intermediate of the padded rows, then the plan
  const bool planned_shapes = a.sh_ranks % 32 == 0 && prefill_plan_supported(P, pt->n_patterns) &&
                              prefill_planned_supported(L->n, L->m, rS);
  const int cap = planned_shapes ? prefill_plan_capacity(rows, P, pt->n_patterns) : 0;
  const size_t zb = planned_shapes ? prefill_planned_z_bytes(cap, rS, prefill_planned_split(rows, L->n)) : 0;
  const bool can_plan = planned_shapes && workspace != nullptr &&
                        workspace_bytes >= zb + prefill_plan_bytes(rows, P, pt->n_patterns);
  if (schedule == PARSE_SCHED_PLANNED && !can_plan) return planned_shapes ? PARSE_EWORKSPACE : PARSE_ESHAPE;
  if (can_plan && (schedule == PARSE_SCHED_PLANNED || schedule == PARSE_SCHED_AUTO)) {
    int32_t *plan = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(workspace) + zb);
    int st = build_prefill_plan(tok_offsets, pattern_id, P, rows, pt->n_patterns, plan, s);
    if (st != PARSE_OK) return st;
    return forward_prefill_planned_bf16(a, plan, cap, (uint16_t *)workspace, rows / (P > 0 ? P : 1), s);
  }
  // two launches of the register-operand tile kernel
  const bool can_split = workspace != nullptr && workspace_bytes >= prefill_split_workspace_bytes(rows, rS) &&
                         prefill_split_supported(L->n, rS);
  bool split = can_split;
  if (schedule == PARSE_SCHED_FUSED) {
    if (a.sh_ranks > 0) return PARSE_ELAYOUT;   // the fused kernel reads one block per pattern
    split = false;
  }
  if (schedule == PARSE_SCHED_TILES || a.sh_ranks > 0) {
    if (!can_split) return prefill_split_supported(L->n, rS) ? PARSE_EWORKSPACE : PARSE_ESHAPE;
    split = true;
  }
  if (split) return forward_prefill_split_bf16(a, (uint16_t *)workspace, rows / (P > 0 ? P : 1), s);
  int BM = 64;
  if (prefill_lds_bytes(64, rS) > kLdsLimit) BM = 32;
  const size_t lds = prefill_lds_bytes(BM, rS);
  if (lds > kLdsLimit) return PARSE_ESHAPE;
  const bool fast = (L->n % (2 * PF_BK) == 0) && (rS % (16 * PF_DEPTH) == 0) && (L->n / 16 >= PF_DEPTH);
  static bool done[4] = {false, false, false, false};
  if (fast) {
    if (BM == 64) return launch_prefill(prefill_fused<64>, &done[0], a, 64, lds, s);
    return launch_prefill(prefill_fused<32>, &done[1], a, 32, lds, s);
  }
  if (BM == 64) return launch_prefill(prefill_fused_any<64>, &done[2], a, 64, lds, s);
  return launch_prefill(prefill_fused_any<32>, &done[3], a, 32, lds, s);
}

}  // namespace parse
