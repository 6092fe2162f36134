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
// A 64-row block of the flat token axis that spans several prompts is processed once per prompt segment.
#include "common.hpp"

namespace parse {

constexpr int PF_THREADS = 256;
constexpr int PF_BK = 64;            // reduction indices per staged X tile (4 matrix instructions deep)
constexpr int PF_XPAD = 8;           // bf16 of padding per LDS row: keeps 16-byte operand reads conflict-free
constexpr int PF_ZPAD = 8;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int BM>
__global__ __launch_bounds__(PF_THREADS) void prefill_fused(
    const uint16_t *__restrict__ X, const uint16_t *__restrict__ Vt_S, const uint16_t *__restrict__ Ut_S,
    int n_patterns, int rows, int n, int m, int rS, const int32_t *__restrict__ tok_offsets,
    const int32_t *__restrict__ pattern_id, int P, uint16_t *__restrict__ Y) {
  constexpr int NT = BM / 32;  // 32-token blocks per workgroup
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const int zld = rS + PF_ZPAD;
  constexpr int xld = PF_BK + PF_XPAD;
  uint16_t *Zs = lds;                          // [BM][zld]
  uint16_t *Xs = lds + (size_t)BM * zld;       // [2][BM][xld]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, q = lane >> 5;
  const int row0 = blockIdx.x * BM;
  const int row_end = min(row0 + BM, rows);
  const int nkb = n / 16;      // 16-wide reduction blocks of phase 1
  const int nrb = rS / 32;     // 32-rank blocks
  const int ncb = m / 32;      // 32-column blocks of the output
  const int nkt = (n + PF_BK - 1) / PF_BK;

  int seg_lo = row0;
  while (seg_lo < row_end) {
    const int p = prompt_of_row(tok_offsets, P, seg_lo);
    int seg_hi = (p + 1 < P) ? tok_offsets[p + 1] : rows;
    seg_hi = min(max(seg_hi, seg_lo + 1), row_end);
    const int pid = pattern_id[p];
    const bool valid = pid >= 0 && pid < n_patterns;
    const uint16_t *Vp = Vt_S + (valid ? (size_t)pid * rS * n : 0);
    const uint16_t *Up = Ut_S + (valid ? (size_t)pid * rS * m : 0);

    // ------------------------------------------------------------ phase 1: Z = X Vt_S^T  -> LDS
    // wave w owns rank blocks w, w+4, w+8, ...; a pass handles up to 4 of them
    const int my_nrb = (nrb - wave + 3) / 4;
    const int passes1 = (nrb + 15) / 16;
    for (int pass = 0; pass < passes1; ++pass) {
      const int nb = max(0, min(4, my_nrb - pass * 4));
      f32x16 acc[NT][4];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[t][i][e] = 0.f;
      // operand base of this wave's i-th rank block: rb = (pass*4 + i)*4 + wave
      const uint16_t *vbase[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rb = min((pass * 4 + i) * 4 + wave, nrb - 1);
        vbase[i] = Vp + ((size_t)rb * nkb * 64 + lane) * 8;
      }
      __syncthreads();  // previous users of Xs (and of Zs in an earlier segment) are done
      // stage X tile 0
      auto load_x = [&](int kt, u32x4 *regs) {
#pragma unroll
        for (int i = 0; i < BM * PF_BK / 8 / PF_THREADS; ++i) {
          const int piece = i * PF_THREADS + threadIdx.x;  // 16-byte piece of the BM x 64 tile
          const int r = piece / (PF_BK / 8), c = (piece % (PF_BK / 8)) * 8;
          const int gr = min(row0 + r, rows - 1);
          const int gc = kt * PF_BK + c;
          regs[i] = (gc < n) ? *reinterpret_cast<const u32x4 *>(X + (size_t)gr * n + gc) : u32x4{0, 0, 0, 0};
        }
      };
      auto store_x = [&](int buf, const u32x4 *regs) {
#pragma unroll
        for (int i = 0; i < BM * PF_BK / 8 / PF_THREADS; ++i) {
          const int piece = i * PF_THREADS + threadIdx.x;
          const int r = piece / (PF_BK / 8), c = (piece % (PF_BK / 8)) * 8;
          *reinterpret_cast<u32x4 *>(Xs + ((size_t)buf * BM + r) * xld + c) = regs[i];
        }
      };
      auto load_v = [&](int kt, u32x4 (*regs)[4]) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const int kb = min(kt * 4 + s, nkb - 1);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (i < nb) regs[s][i] = *reinterpret_cast<const u32x4 *>(vbase[i] + (size_t)kb * 512);
        }
      };
      u32x4 xr[BM * PF_BK / 8 / PF_THREADS];
      u32x4 va[4][4], vb[4][4];
      load_x(0, xr);
      load_v(0, va);
      store_x(0, xr);
      __syncthreads();
      for (int kt = 0; kt < nkt; ++kt) {
        const int buf = kt & 1;
        const bool more = kt + 1 < nkt;
        if (more) {
          load_x(kt + 1, xr);
          load_v(kt + 1, vb);
        }
        const int ksteps = min(4, nkb - kt * 4);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          if (s < ksteps) {
            bf16x8 xb[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t)
              xb[t] = as_bf16x8(*reinterpret_cast<const u32x4 *>(Xs + ((size_t)buf * BM + t * 32 + l32) * xld + s * 16 + q * 8));
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (i < nb) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
                  acc[t][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va[s][i]), xb[t], acc[t][i], 0, 0, 0);
              }
          }
        }
        if (more) {
          store_x(buf ^ 1, xr);
#pragma unroll
          for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i) va[s][i] = vb[s][i];
        }
        __syncthreads();
      }
      // accumulators -> bf16 -> Z block.  lane holds token l32 of block t, ranks rb*32 + 8*blk + 4*q + (0..3)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i < nb) {
          const int rb = (pass * 4 + i) * 4 + wave;
#pragma unroll
          for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
              u32x2 w;
              w[0] = pack_bf16x2(acc[t][i][blk * 4 + 0], acc[t][i][blk * 4 + 1]);
              w[1] = pack_bf16x2(acc[t][i][blk * 4 + 2], acc[t][i][blk * 4 + 3]);
              *reinterpret_cast<u32x2 *>(Zs + (size_t)(t * 32 + l32) * zld + rb * 32 + blk * 8 + q * 4) = w;
            }
        }
    }
    __syncthreads();  // Z block complete

    // ------------------------------------------------------------ phase 2: Y = Z Ut_S
    const int nk2 = rS / 16;
    const int passes2 = (ncb + 15) / 16;
    for (int pass = 0; pass < passes2; ++pass) {
      const int cb0 = pass * 16 + wave * 4;
      const int nb = max(0, min(4, ncb - cb0));
      if (nb == 0) continue;   // no barriers below: a wave may skip
      f32x16 acc[NT][4];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[t][i][e] = 0.f;
      const uint16_t *ubase = Up + ((size_t)cb0 * 64 + lane) * 8;   // + kb * ncb * 512 + i * 512
      auto load_u = [&](int kb, u32x4 *regs) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (i < nb) regs[i] = *reinterpret_cast<const u32x4 *>(ubase + ((size_t)kb * ncb + i) * 512);
      };
      constexpr int DEPTH = 4;
      u32x4 ua[DEPTH][4];
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) load_u(min(d, nk2 - 1), ua[d]);
      for (int kb0 = 0; kb0 < nk2; kb0 += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
          const int kb = kb0 + d;
          if (kb < nk2) {
            bf16x8 zb[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t)
              zb[t] = as_bf16x8(*reinterpret_cast<const u32x4 *>(Zs + (size_t)(t * 32 + l32) * zld + kb * 16 + q * 8));
            u32x4 cur[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) cur[i] = ua[d][i];
            load_u(min(kb + DEPTH, nk2 - 1), ua[d]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (i < nb) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
                  acc[t][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(cur[i]), zb[t], acc[t][i], 0, 0, 0);
              }
          }
        }
      }
      // store: lane holds token t*32 + l32, columns (cb0+i)*32 + 8*blk + 4*q + (0..3)
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int r = row0 + t * 32 + l32;
        if (r < seg_lo || r >= seg_hi) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (i < nb) {
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
              u32x2 w;
              if (valid) {
                w[0] = pack_bf16x2(acc[t][i][blk * 4 + 0], acc[t][i][blk * 4 + 1]);
                w[1] = pack_bf16x2(acc[t][i][blk * 4 + 2], acc[t][i][blk * 4 + 3]);
              } else {
                w[0] = 0; w[1] = 0;
              }
              *reinterpret_cast<u32x2 *>(Y + (size_t)r * m + (cb0 + i) * 32 + blk * 8 + q * 4) = w;
            }
          }
      }
    }
    seg_lo = seg_hi;
  }
}

size_t prefill_lds_bytes(int BM, int rS) {
  return ((size_t)BM * (rS + PF_ZPAD) + 2 * (size_t)BM * (PF_BK + PF_XPAD)) * sizeof(uint16_t);
}

constexpr size_t kLdsLimit = 160 * 1024;

int forward_prefill_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *X, int rows,
                         const int32_t *tok_offsets, const int32_t *pattern_id, int P, uint16_t *Y, hipStream_t s) {
  const int gs = L->R / L->G, rS = pt->k * gs;
  int BM = 64;
  if (prefill_lds_bytes(64, rS) > kLdsLimit) BM = 32;
  const size_t lds = prefill_lds_bytes(BM, rS);
  if (lds > kLdsLimit) return PARSE_ESHAPE;
  const dim3 grid((rows + BM - 1) / BM);
  if (BM == 64) {
    static bool attr64 = false;
    if (!attr64) {
      PARSE_HIP_TRY(hipFuncSetAttribute((const void *)prefill_fused<64>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)kLdsLimit));
      attr64 = true;
    }
    hipLaunchKernelGGL(prefill_fused<64>, grid, dim3(PF_THREADS), lds, s, X, (const uint16_t *)pt->Vt_S,
                       (const uint16_t *)pt->Ut_S, pt->n_patterns, rows, L->n, L->m, rS, tok_offsets, pattern_id, P, Y);
  } else {
    static bool attr32 = false;
    if (!attr32) {
      PARSE_HIP_TRY(hipFuncSetAttribute((const void *)prefill_fused<32>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)kLdsLimit));
      attr32 = true;
    }
    hipLaunchKernelGGL(prefill_fused<32>, grid, dim3(PF_THREADS), lds, s, X, (const uint16_t *)pt->Vt_S,
                       (const uint16_t *)pt->Ut_S, pt->n_patterns, rows, L->n, L->m, rS, tok_offsets, pattern_id, P, Y);
  }
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // namespace parse
