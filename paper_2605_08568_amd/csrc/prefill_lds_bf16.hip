// a6, planned form of the bf16 prefill product (Sec. 4.4, Eq. 10):  launch 1  Z = X Vt_S^T,  launch 2  Y = Z Ut_S,
// both with ONE tile kernel, `gemm_lds`, over the virtual rows of a prefill plan (plan.hip): a tile of token rows
// belongs to one pattern, so a workgroup runs one reduction with one factor block, whatever the prompt lengths.
//
// Data path.  Both operands of a tile are staged in LDS by loads that write LDS directly (no register round trip,
// 1 KiB per wavefront instruction), STAGES reduction slices of BK deep; the matrix-core operands are then 16-byte
// LDS reads.  Factor operands are stored in operand order in memory (PARSE_MFMA16), so a 1 KiB load lands as one
// ready operand and is read back linearly (conflict-free).  The intermediate Z is written by launch 1 in the same
// operand order (token block x reduction block), so launch 2 stages it exactly like a factor.  Only X is row-major:
// its rows are loaded 16 bytes per lane, whole cache lines per row, and the 16-byte chunks of a row are XOR-swizzled
// on the way in (the swizzle is applied to the global address, the LDS write is linear) so that the operand reads --
// 32 rows x one chunk -- spread over all banks.
// Pipeline per reduction slice: ... [LDS reads of step s+1 | matrix instructions of step s] ...; in the last step of
// a slice the wavefront waits for its own loads of the next slice, meets the others at a barrier (so everybody's loads
// have landed and everybody is done reading the current slice), requests the slice STAGES ahead into the buffer just
// freed and reads the next slice's first operands -- all of that while its matrix instructions of the last step are
// still to be issued, so the matrix pipe does not drain at the barrier.
// Output: the accumulator of the 32x32x16 instruction gives a lane 4 consecutive factor rows (output columns) of one
// token in each of four 8-row bands; one 32-lane swap pairs the bands up to 8 consecutive columns = 16 bytes, which is
// one piece of a Z operand (launch 1: stored linearly, 1 KiB per instruction) or a 16-byte store into the token's
// row of Y (launch 2).
#include <algorithm>

#include "prefill_common.hpp"

namespace parse {

#define PARSE_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define PARSE_GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

template <int N> __device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit count");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// barrier without the fences of __syncthreads(): those would wait for ALL outstanding loads, also the slices
// requested ahead.  The explicit vmcnt wait before it covers exactly the slice that is about to be read.
__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

constexpr int LG_MAX_LAYERS = 4;

// One product of one layer.  A launch covers up to LG_MAX_LAYERS of them (layers that share their token rows and the
// plan: the stacked first product and the batched second product of Sec. 4.4, Eq. 11-12): the column tiles of the
// layers are numbered through, tn_first is a layer's first.
struct LgLayer {
  const uint16_t *Tk;      // TROW 1: row-major [rows][K] (X);  TROW 0: Z in operand order [(virtual rows)/32][K/16][1 KiB]
  const uint16_t *F;       // factor operands of all patterns
  uint16_t *O;             // OROW 0: Z (operand order);  OROW 1: Y row-major [rows][M]
  float *Pz;               // SPLIT: fp32 partial sums of Z, [slice][token block][reduction block][64 lanes][8]
  size_t pattern_stride;   // elements of F per pattern
  int K, M;                // reduction length, factor rows (= output columns)
  // shared head (Sec. 4.4: shared experts at the head of memory, stored once): the first sh_blocks 32-rank blocks of
  // every pattern's selection come from Fsh (same operand order, as many rank rows as the head has), the per-pattern
  // blocks in F hold the rest, renumbered from 0.  FORD 0: the leading factor-row blocks; FORD 1 (BK == 32 only): the
  // leading reduction slices.  0 = everything per pattern.
  const uint16_t *Fsh;
  int sh_blocks;
  int tn_first;            // first column tile of this layer in the launch
};
struct LgArgs {
  LgLayer L[LG_MAX_LAYERS];
  int n_layers;
  const int32_t *plan;     // header | tile patterns | row map (plan.hip)
  int cap;                 // plan capacity in 256-row tiles (fixes where the row map starts)
  int ntn, gm, ngroups;    // column tiles (all layers), token tiles per locality group, groups
  int ks;                  // SPLIT: slices of the reduction range, one workgroup each
};

// FORD: factor order, 0 = right factor (operand (rb, kb) at rb*(K/16)+kb), 1 = left factor (operand (kb, cb) at kb*(M/32)+cb).
// TROW: token operand 1 = row-major rows looked up through the plan's row map (X, or a row-major intermediate),
//       0 = operand order over the plan's virtual rows.   OROW: output 1 = row-major through the row map, 0 = operand order.
// First product: <FORD 0, TROW 1, OROW 0>; second product: <FORD 1, TROW 0, OROW 1>.
// SPLIT (first product only): the reduction range is cut in a.ks slices, one workgroup each; a workgroup stores its fp32
// sums as slice s of the partial sums and z_combine adds the slices (in slice order) and rounds -- for launches whose
// tiles alone would leave most compute units idle (one short prompt).
template <int BM, int BN, int WM, int WN, int BK, int STAGES, int FORD, int TROW, int OROW, int SPLIT = 0>
__global__ __launch_bounds__(WM * WN * 64) void gemm_lds(LgArgs a) {
  static_assert(!SPLIT || (FORD == 0 && OROW == 0), "only the first product is split");
  constexpr int NW = WM * WN;
  constexpr int KK = BK / 16;                 // matrix-instruction steps per staged slice
  constexpr int TB = BM / WM / 32, FB = BN / WN / 32;
  constexpr int F_BYTES = BN * BK * 2, T_BYTES = BM * BK * 2, STAGE_BYTES = F_BYTES + T_BYTES;
  constexpr int NI_F = F_BYTES / 1024, NI_T = T_BYTES / 1024;   // 1 KiB load instructions per slice
  static_assert(NI_F % NW == 0 && NI_T % NW == 0, "the loads of a slice divide evenly over the wavefronts");
  static_assert(KK == 2 || KK == 4, "register double-buffering assumes an even number of steps");
  static_assert(256 % BM == 0, "token tiles subdivide the plan's 256-row tiles");
  constexpr int LF = NI_F / NW, LT = NI_T / NW, L = LF + LT;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int j = lane & 31, q = lane >> 5;

  // tile of this workgroup: consecutive ids share a die (and its L2); within a locality group the token tile runs fastest
  // The grid is sized for the plan's capacity; the real tile count comes from the plan.  Workgroups past it leave at
  // once, the others are renumbered over the REAL count so that every die gets its share.
  const int per = a.gm * a.ntn;
  const int vrows = a.plan[1];
  const int n_real = ((vrows + BM - 1) / BM + a.gm - 1) / a.gm * per;
  const int ks = SPLIT ? a.ks : 1;
  const int bid = SPLIT ? (int)blockIdx.x / ks : (int)blockIdx.x, sl = SPLIT ? (int)blockIdx.x % ks : 0;
  if (bid >= n_real) return;
  const int tile = xcd_tile(bid, n_real);
  const int g = tile / per, r = tile % per;
  const int tm = g * a.gm + r % a.gm;
  int tn = r / a.gm;                           // column tile over all layers of the launch
  int li = 0;
#pragma unroll
  for (int i = 1; i < LG_MAX_LAYERS; ++i) li += (i < a.n_layers && tn >= a.L[i].tn_first) ? 1 : 0;
  const LgLayer &ly = a.L[li];
  tn -= ly.tn_first;
  const int K = ly.K, M = ly.M;
  const int kt0 = SPLIT ? (int)(((long long)(K / BK) * sl) / ks) : 0;           // first slice of BK of this workgroup
  const int nk = (SPLIT ? (int)(((long long)(K / BK) * (sl + 1)) / ks) : K / BK) - kt0;
  if (tm * BM >= vrows) return;                // the last locality group may be partial
  const int32_t *tile_pat = a.plan + 16;
  const int32_t *rowmap = a.plan + 16 + (a.cap + 15) / 16 * 16;
  const int pat = tile_pat[tm * BM / 256];
  if (pat < 0) {
    // prompts without a valid pattern: the first product has nothing to do, the second one writes zero rows
    if (OROW == 1 && FORD == 1) {
      for (int rr = wave; rr < BM; rr += NW) {
        const int orow = rowmap[tm * BM + rr];
        if (orow < 0) continue;
        for (int c = lane * 8; c < BN; c += 512) {
          const int col = tn * BN + c;
          if (col < M) *reinterpret_cast<u32x4 *>(ly.O + (size_t)orow * M + col) = u32x4{0, 0, 0, 0};
        }
      }
    }
    return;
  }
  const uint16_t *Fp = ly.F + (size_t)pat * ly.pattern_stride;

  // ---- per-lane global sources of this wavefront's load instructions; they advance by a constant per slice ----
  const char *fsrc[LF];
  const char *fsrc_own[LF];                    // FORD 1 with a shared head: where the pattern's own slices start
  int fdst[LF];
  const int shb = ly.sh_blocks;
#pragma unroll
  for (int i = 0; i < LF; ++i) {
    const int ins = wave + i * NW;             // instruction id within the factor part, LDS order [fb][kk]
    const int fb = ins / KK, kk = ins % KK;
    const int gb = min(tn * (BN / 32) + fb, M / 32 - 1);   // blocks past the end re-read the last one (never stored)
    if (FORD == 0) {
      const char *src = gb < shb ? (const char *)ly.Fsh + (size_t)gb * (K / 16) * 1024
                                 : (const char *)Fp + (size_t)(gb - shb) * (K / 16) * 1024;
      fsrc[i] = src + (size_t)kk * 1024 + lane * 16;
      fsrc_own[i] = fsrc[i];
    } else {
      fsrc_own[i] = (const char *)Fp + ((size_t)kk * (M / 32) + gb) * 1024 + lane * 16;
      fsrc[i] = shb > 0 ? (const char *)ly.Fsh + ((size_t)kk * (M / 32) + gb) * 1024 + lane * 16 : fsrc_own[i];
    }
    fdst[i] = ins * 1024;
  }
  const size_t fstep = FORD == 0 ? (size_t)KK * 1024 : (size_t)KK * (M / 32) * 1024;
  int issued = 0;                              // FORD 1: slices requested so far (a slice of BK = 32 is one 32-rank block)
  const char *tsrc[LT];
  int tdst[LT];
  constexpr int CPR = BK * 2 / 16;             // 16-byte chunks per staged X row
#pragma unroll
  for (int i = 0; i < LT; ++i) {
    const int ins = wave + i * NW;
    if (TROW == 0) {
      const int tb = ins / KK, kk = ins % KK;
      tsrc[i] = (const char *)ly.Tk + ((size_t)(tm * (BM / 32) + tb) * (K / 16) + kk) * 1024 + lane * 16;
    } else {
      constexpr int RPI = 1024 / (BK * 2);     // rows per instruction
      const int rr = ins * RPI + lane / CPR, cp = lane % CPR;   // LDS position (row, chunk slot)
      const int sw = CPR == 4 ? ((rr >> 2) & 3) : ((rr >> 1) & 7);
      const int c = cp ^ sw;                                    // chunk of the row that is stored in that slot
      int row = rowmap[tm * BM + rr];
      row = row < 0 ? 0 : row;                 // padding rows read row 0; their results are never stored to Y
      tsrc[i] = (const char *)ly.Tk + (size_t)row * K * 2 + c * 16;
    }
    tdst[i] = F_BYTES + ins * 1024;
  }
  const size_t tstep = TROW == 0 ? (size_t)KK * 1024 : (size_t)BK * 2;
  if (SPLIT) {
#pragma unroll
    for (int i = 0; i < LF; ++i) { fsrc[i] += (size_t)kt0 * fstep; fsrc_own[i] = fsrc[i]; }
#pragma unroll
    for (int i = 0; i < LT; ++i) tsrc[i] += (size_t)kt0 * tstep;
  }

  auto issue = [&](int stage_buf) {
    char *base = smem + stage_buf * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < LF; ++i) {
      __builtin_amdgcn_global_load_lds(PARSE_GLB_PTR(fsrc[i]), PARSE_LDS_PTR(base + fdst[i]), 16, 0, 0);
      fsrc[i] += fstep;
    }
#pragma unroll
    for (int i = 0; i < LT; ++i) {
      __builtin_amdgcn_global_load_lds(PARSE_GLB_PTR(tsrc[i]), PARSE_LDS_PTR(base + tdst[i]), 16, 0, 0);
      tsrc[i] += tstep;
    }
    if (FORD == 1 && BK == 32) {               // the reduction leaves the shared head: continue in the pattern's own block
      if (++issued == shb) {
#pragma unroll
        for (int i = 0; i < LF; ++i) fsrc[i] = fsrc_own[i];
      }
    }
  };

  // ---- LDS operand addresses (relative to the slice's buffer) ----
  int foff[FB], toff[TB];
#pragma unroll
  for (int i = 0; i < FB; ++i) foff[i] = ((wn * FB + i) * KK) * 1024 + lane * 16;
#pragma unroll
  for (int t = 0; t < TB; ++t) {
    if (TROW == 0) toff[t] = F_BYTES + ((wm * TB + t) * KK) * 1024 + lane * 16;
    else toff[t] = F_BYTES + (wm * TB * 32 + t * 32 + j) * (BK * 2);
  }
  auto tchunk = [&](int t, int kk) -> int {    // byte offset of this lane's 16 bytes of token operand (t, kk)
    if (TROW == 0) return toff[t] + kk * 1024;
    const int rr = wm * TB * 32 + t * 32 + j;
    const int sw = CPR == 4 ? ((rr >> 2) & 3) : ((rr >> 1) & 7);
    return toff[t] + (((kk * 2 + q) ^ sw) * 16);
  };

  f32x16 acc[TB][FB];
#pragma unroll
  for (int t = 0; t < TB; ++t)
#pragma unroll
    for (int i = 0; i < FB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][i][e] = 0.f;

  u32x4 fr[2][FB], tr[2][TB];
  auto read_ops = [&](int buf, int stage_buf, int kk) {
    const char *base = smem + stage_buf * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < FB; ++i) fr[buf][i] = *reinterpret_cast<const u32x4 *>(base + foff[i] + kk * 1024);
#pragma unroll
    for (int t = 0; t < TB; ++t) tr[buf][t] = *reinterpret_cast<const u32x4 *>(base + tchunk(t, kk));
  };

  // The compiler treats a load that writes LDS directly like a flat access that may complete out of order with LDS
  // reads, so after one of them every wait it inserts for LDS data is a wait for ALL outstanding LDS reads.  Placed by
  // the compiler that wait sits between the reads of the next step and the matrix instructions of this step and exposes
  // the LDS latency once per slice.  Touching this step's operands BEFORE the next step's reads are issued moves the wait
  // to where nothing is outstanding but reads that had a whole step to finish.
  auto settle = [&](int buf) {
#pragma unroll
    for (int i = 0; i < FB; ++i) asm volatile("" ::"v"(fr[buf][i]));
#pragma unroll
    for (int t = 0; t < TB; ++t) asm volatile("" ::"v"(tr[buf][t]));
  };

  // prologue: STAGES-1 slices requested, the first one awaited, one more requested
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nk) issue(s);
  if (nk >= STAGES - 1) wait_vm<(STAGES - 2) * L>(); else wait_vm<0>();
  wg_barrier();
  if (STAGES - 1 < nk) issue((STAGES - 1) % STAGES);
  read_ops(0, 0, 0);

  for (int kt = 0; kt < nk; ++kt) {
    const int sb = kt % STAGES;
#pragma unroll
    for (int s = 0; s < KK; ++s) {
      const int cur = s & 1;
      settle(cur);
      __builtin_amdgcn_sched_barrier(0);
      if (s < KK - 1) {
        read_ops(cur ^ 1, sb, s + 1);
      } else if (kt + 1 < nk) {
        // hand-over: slice kt+1 must have landed for every wavefront; slice kt's buffer is free after the barrier
        const int later = min(kt + STAGES - 1, nk - 1) - (kt + 1);   // slices requested after kt+1
        if (later >= STAGES - 2) wait_vm<(STAGES - 2) * L>();
        else if (STAGES > 3 && later == 1) wait_vm<L>();
        else wait_vm<0>();
        wg_barrier();
        if (kt + STAGES < nk) issue(sb);
        read_ops(cur ^ 1, (kt + 1) % STAGES, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < FB; ++i)
#pragma unroll
        for (int t = 0; t < TB; ++t)
          acc[t][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fr[cur][i]), as_bf16x8(tr[cur][t]), acc[t][i], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- output: lane (j, q) of acc[t][i] holds token t*32+j, factor rows i*32 + 8*band + 4*q + (0..3) ----
#pragma unroll
  for (int t = 0; t < TB; ++t) {
    const int vrow = tm * BM + (wm * TB + t) * 32 + j;
    int orow = -1;
    if (OROW == 1) orow = rowmap[vrow];
#pragma unroll
    for (int i = 0; i < FB; ++i) {
      const int gb = tn * (BN / 32) + wn * FB + i;     // 32-row factor block of the whole matrix
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (SPLIT) {   // the same exchange on the fp32 sums: lane (j, q) ends up with the 8 consecutive factor rows of its token
          float w8[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[t][i][(2 * h) * 4 + e]),
                                                             __float_as_uint(acc[t][i][(2 * h + 1) * 4 + e]), false, false);
            w8[e] = __uint_as_float(sw[0]); w8[4 + e] = __uint_as_float(sw[1]);
          }
          if (gb < M / 32) {
            const int tbg = tm * (BM / 32) + wm * TB + t;
            float *dst = ly.Pz + (((size_t)sl * (a.cap * 8) + tbg) * (M / 16) + gb * 2 + h) * 512 + lane * 8;
            *reinterpret_cast<float4 *>(dst) = float4{w8[0], w8[1], w8[2], w8[3]};
            *reinterpret_cast<float4 *>(dst + 4) = float4{w8[4], w8[5], w8[6], w8[7]};
          }
          continue;
        }
        const uint32_t p0x = cvt_pk_bf16(acc[t][i][(2 * h) * 4 + 0], acc[t][i][(2 * h) * 4 + 1]);
        const uint32_t p0y = cvt_pk_bf16(acc[t][i][(2 * h) * 4 + 2], acc[t][i][(2 * h) * 4 + 3]);
        const uint32_t p1x = cvt_pk_bf16(acc[t][i][(2 * h + 1) * 4 + 0], acc[t][i][(2 * h + 1) * 4 + 1]);
        const uint32_t p1y = cvt_pk_bf16(acc[t][i][(2 * h + 1) * 4 + 2], acc[t][i][(2 * h + 1) * 4 + 3]);
        // the upper 32 lanes of band 2h are exchanged with the lower 32 lanes of band 2h+1: afterwards lane (j, q)
        // holds the 8 consecutive factor rows gb*32 + 16h + 8q + (0..7) of its token
        const u32x2 sx = __builtin_amdgcn_permlane32_swap(p0x, p1x, false, false);
        const u32x2 sy = __builtin_amdgcn_permlane32_swap(p0y, p1y, false, false);
        const u32x4 w = {sx[0], sy[0], sx[1], sy[1]};
        if (gb < M / 32) {
          if (OROW == 0) {   // Z operand (token block, reduction block gb*2 + h), lane's piece at lane*16
            const int tbg = tm * (BM / 32) + wm * TB + t;
            *reinterpret_cast<u32x4 *>((char *)ly.O + ((size_t)tbg * (M / 16) + gb * 2 + h) * 1024 + lane * 16) = w;
          } else if (orow >= 0) {
            *reinterpret_cast<u32x4 *>(ly.O + (size_t)orow * M + gb * 32 + h * 16 + q * 8) = w;
          }
        }
      }
    }
  }
}

// Adds the ks partial sums of every 16-byte piece of Z (8 consecutive ranks of a token) in slice order and rounds to
// bf16.  One thread per piece, over the plan's virtual rows (pieces of tiles without a pattern hold nothing and are not
// read by the second product either).
__global__ __launch_bounds__(256) void z_combine(const float *__restrict__ Pz, int ks, int cap, int M, const int32_t *__restrict__ plan,
                                                 uint16_t *__restrict__ Z) {
  const size_t pieces = (size_t)(plan[1] / 32) * (M / 16) * 64;      // virtual rows / 32 token blocks x reduction blocks x lanes
  const size_t slice = (size_t)cap * 8 * (M / 16) * 512;             // floats per slice
  for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < pieces; o += (size_t)gridDim.x * 256) {
    const float *src = Pz + o * 8;
    float4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < ks; s0 += 4) {      // four slices requested at a time (slices past the last re-read it)
      float4 l4[4], h4[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float *ps = src + (size_t)min(s0 + u, ks - 1) * slice;
        l4[u] = *reinterpret_cast<const float4 *>(ps);
        h4[u] = *reinterpret_cast<const float4 *>(ps + 4);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (s0 + u < ks) {
          lo.x += l4[u].x; lo.y += l4[u].y; lo.z += l4[u].z; lo.w += l4[u].w;
          hi.x += h4[u].x; hi.y += h4[u].y; hi.z += h4[u].z; hi.w += h4[u].w;
        }
      }
    }
    *reinterpret_cast<u32x4 *>(Z + o * 8) =
        u32x4{cvt_pk_bf16(lo.x, lo.y), cvt_pk_bf16(lo.z, lo.w), cvt_pk_bf16(hi.x, hi.y), cvt_pk_bf16(hi.z, hi.w)};
  }
}

template <int BM, int BN, int WM, int WN, int BK, int STAGES, int FORD, int TROW, int OROW, int SPLIT = 0>
static int launch_gemm_lds(LgArgs a, int avg_tiles_per_pattern, hipStream_t s) {
  constexpr int smem = STAGES * (BM + BN) * BK * 2;
  auto kern = gemm_lds<BM, BN, WM, WN, BK, STAGES, FORD, TROW, OROW, SPLIT>;
  static bool attr_done[64] = {false};
  int dev = 0;
  PARSE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return PARSE_EINVAL;
  if (!attr_done[dev]) {
    PARSE_HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem));
    attr_done[dev] = true;
  }
  const int ntm = a.cap * (256 / BM);          // token tiles the plan can hold (the kernel exits past the real count)
  a.ntn = 0;
  for (int l = 0; l < a.n_layers; ++l) {
    a.L[l].tn_first = a.ntn;
    a.ntn += (a.L[l].M + BN - 1) / BN;
  }
  int gm = avg_tiles_per_pattern * (256 / BM);
  a.gm = gm < 1 ? 1 : (gm > 8 ? 8 : gm);
  a.ngroups = (ntm + a.gm - 1) / a.gm;
  hipLaunchKernelGGL(kern, dim3(a.ngroups * a.gm * a.ntn * (SPLIT ? a.ks : 1)), dim3(WM * WN * 64), smem, s, a);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

// Z workspace of the planned form: the plan's capacity in virtual rows x rS bf16 (operand order)
// Slices of the first product's reduction range (1 = no split): only for batches of at most 1024 token rows (16 tiles
// of 64 tokens: with the eight or so 128-rank tiles of a selection they leave half of the compute units without a
// workgroup), as many as bring the token tiles x slices to 32, at most 8, at least 8 staged slices of 64 per workgroup.
// A function of (rows, n) alone, so that a call over several layers splits exactly like its single-layer calls and
// gives the same bits.
int prefill_planned_split(int rows, int n) {
  const int tiles = (rows + 63) / 64;
  if (tiles <= 0 || tiles > 16) return 1;
  int ks = 32 / tiles;
  if (ks > 8) ks = 8;
  if (ks > n / 64 / 8) ks = n / 64 / 8;
  return ks < 2 ? 1 : ks;
}
// Z of one layer (bf16, operand order over the plan's capacity), then -- when the first product is split -- the fp32
// partial sums of its ks slices
static size_t planned_z_only_bytes(int cap_tiles, int rS) { return round_up((size_t)cap_tiles * 256 * rS * sizeof(uint16_t), 256); }
size_t prefill_planned_z_bytes(int cap_tiles, int rS, int ks) {
  return planned_z_only_bytes(cap_tiles, rS) + (ks > 1 ? round_up((size_t)ks * cap_tiles * 256 * rS * sizeof(float), 256) : 0);
}

bool prefill_planned_supported(int n, int m, int rS) { return n % 64 == 0 && rS % 32 == 0 && m % 32 == 0 && n >= 64 && rS >= 32; }

// n_layers layers that share X [rows][n] (row-major) and the plan (built for the tok_offsets and pattern ids of these
// patterns); Z[l] = layer l's intermediate (operand order over the plan's virtual rows); p[l].Y [rows][m_l].
// Two launches for all layers together: the stacked first product, the batched second product (Sec. 4.4, Eq. 11-12).
int forward_prefill_planned_multi_bf16(const PfArgs *p, int n_layers, const int32_t *plan, int cap, uint16_t *const *Z,
                                       int avg_prompt_rows, hipStream_t s) {
  if (n_layers < 1 || n_layers > LG_MAX_LAYERS) return PARSE_ESHAPE;
  LgArgs g1{}, g2{};
  g1.n_layers = g2.n_layers = n_layers;
  g1.plan = g2.plan = plan;
  g1.cap = g2.cap = cap;
  long long ct1 = 0, ct2 = 0;                  // 256-wide column tiles of the two products, all layers
  for (int l = 0; l < n_layers; ++l) {
    if (p[l].sh_ranks % 32 != 0 || p[l].sh_ranks >= p[l].rS) return PARSE_ESHAPE;
    const int own = p[l].rS - p[l].sh_ranks;   // ranks in a pattern's own block
    g1.L[l] = LgLayer{p[l].X, p[l].Vt_S, Z[l], nullptr, (size_t)own * p[l].n, p[l].n, p[l].rS, p[l].Vt_sh, p[l].sh_ranks / 32, 0};
    g2.L[l] = LgLayer{Z[l], p[l].Ut_S, p[l].Y, nullptr, (size_t)own * p[l].m, p[l].rS, p[l].m, p[l].Ut_sh, p[l].sh_ranks / 32, 0};
    ct1 += (p[l].rS + 255) / 256;
    ct2 += (p[l].m + 255) / 256;
  }
  const long long tiles256 = (long long)((p[0].rows + 255) / 256);
  const int per_pattern = avg_prompt_rows / 256;
  // 256 x 256 tiles halve the bytes a compute unit has to take in per flop; they are used when they still give the
  // chip enough workgroups, 128 x 128 tiles otherwise (config 1's first product: 64 large tiles or 256 small ones)
  const bool big1 = tiles256 * ct1 >= 192;
  const bool big2 = tiles256 * ct2 >= 192;
  // a product that does not even fill the chip with 128 x 128 tiles (one long prompt through a narrow selection:
  // 2048 tokens x 1024 ranks are 128 tiles for 256 compute units) takes 64-token tiles: more bytes per flop for a unit,
  // but twice the units at work
  long long t128 = 0;
  for (int l = 0; l < n_layers; ++l) t128 += (long long)((p[0].rows + 127) / 128) * ((p[l].rS + 127) / 128);
  const bool small1 = !big1 && t128 <= 192;
  const int ks = small1 ? prefill_planned_split(p[0].rows, p[0].n) : 1;
  if (ks > 1) {      // the partial sums follow each layer's Z in the workspace
    g1.ks = ks;
    for (int l = 0; l < n_layers; ++l)
      g1.L[l].Pz = reinterpret_cast<float *>(reinterpret_cast<char *>(Z[l]) + planned_z_only_bytes(cap, p[l].rS));
  }
  long long u128 = 0;                          // the same for the second product
  for (int l = 0; l < n_layers; ++l) u128 += (long long)((p[0].rows + 127) / 128) * ((p[l].m + 127) / 128);
  const bool small2 = !big2 && u128 <= 192;
  int st;
  if (ks > 1) {
    st = launch_gemm_lds<64, 128, 2, 2, 64, 4, 0, 1, 0, 1>(g1, per_pattern, s);
    for (int l = 0; l < n_layers && st == PARSE_OK; ++l) {
      const size_t pieces = (size_t)cap * 8 * (p[l].rS / 16) * 64;
      hipLaunchKernelGGL(z_combine, dim3((unsigned)std::min<size_t>((pieces + 255) / 256, 2048)), dim3(256), 0, s, g1.L[l].Pz, ks, cap,
                         p[l].rS, plan, Z[l]);
      PARSE_LAUNCH_CHECK();
    }
  } else if (big1) st = launch_gemm_lds<256, 256, 2, 2, 32, 4, 0, 1, 0>(g1, per_pattern, s);
  else if (small1) st = launch_gemm_lds<64, 128, 2, 2, 64, 4, 0, 1, 0>(g1, per_pattern, s);
  else st = launch_gemm_lds<128, 128, 2, 2, 64, 4, 0, 1, 0>(g1, per_pattern, s);
  if (st != PARSE_OK) return st;
  if (big2) return launch_gemm_lds<256, 256, 2, 4, 32, 4, 1, 0, 1>(g2, per_pattern, s);
  if (small2) return launch_gemm_lds<64, 128, 2, 2, 32, 4, 1, 0, 1>(g2, per_pattern, s);
  return launch_gemm_lds<128, 128, 2, 2, 32, 4, 1, 0, 1>(g2, per_pattern, s);
}

int forward_prefill_planned_bf16(const PfArgs &p, const int32_t *plan, int cap, uint16_t *Z, int avg_prompt_rows,
                                 hipStream_t s) {
  uint16_t *Zs[1] = {Z};
  return forward_prefill_planned_multi_bf16(&p, 1, plan, cap, Zs, avg_prompt_rows, s);
}

}  // namespace parse
