// a7: decode step for bf16 PARSE_MFMA16 layers (Sec. 4.3, "Rank Reuse for Decoding"): every sequence keeps the
// rank subset chosen at prefill; one token per sequence.  Bandwidth-bound: the kernels stream each rank group
// that ANY sequence of the batch selected exactly once, straight from the layer's factor store in operand
// order (1 KiB coalesced per wavefront instruction, no LDS hop, no packed copies), and apply it to all
// sequences at once on the matrix cores (32 sequences = the N side of a 32x32x16 instruction).  A sequence
// whose pattern does not hold a group gets a zero in that group's part of z, so it contributes nothing.
//
//   decode_z     z partials: workgroup = (32-rank block, slice of the reduction axis n); 4 wavefronts split
//                the slice and reduce through LDS; skipped entirely if no sequence uses the block's group.
//   decode_zfin  adds the slices in order, masks by pattern membership, rounds to bf16 and lays z out in
//                operand order for phase 2 (tiny).
//   decode_y     workgroup = one 32-column block of the output; 8 wavefronts split the selected ranks,
//                reduce through LDS and store y as bf16.
#include "common.hpp"

namespace parse {

constexpr int DZ_THREADS = 256;
constexpr int DY_THREADS = 512;
constexpr int DEC_DEPTH = 8;   // operand fetches in flight per wavefront
constexpr int DEC_MAXG = 64;

__device__ __forceinline__ bf16x8 dec_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// bit b of the result: sequence b (< B <= 32) holds group g in its pattern
__device__ __forceinline__ bool seq_uses_group(const int32_t *__restrict__ subsets, int stride, int k, int n_patterns,
                                               const int32_t *__restrict__ pattern_id, int B, int b, int g) {
  if (b >= B) return false;
  const int pid = pattern_id[b];
  if (pid < 0 || pid >= n_patterns) return false;
  bool u = false;
  for (int i = 0; i < k; ++i) u = u || (subsets[(size_t)pid * stride + i] == g);
  return u;
}

// grid (R/32, KS)
__global__ __launch_bounds__(DZ_THREADS) void decode_z(const uint16_t *__restrict__ Vt, const uint16_t *__restrict__ x,
                                                       int B, int n, int R, int gs, const int32_t *__restrict__ subsets,
                                                       int stride, int k, int n_patterns,
                                                       const int32_t *__restrict__ pattern_id, int KS,
                                                       float *__restrict__ zp) {
  __shared__ float red[3][16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, q = lane >> 5;
  const int rb = blockIdx.x, ks = blockIdx.y;
  const int g = rb * 32 / gs;
  const bool mine = seq_uses_group(subsets, stride, k, n_patterns, pattern_id, B, l32, g);
  if (__ballot(mine) == 0ull) return;   // nobody selected this group: nothing is read
  const int nkb = n / 16;
  const int w0 = (int)(((long long)nkb * ks) / KS), w1 = (int)(((long long)nkb * (ks + 1)) / KS);
  const int len = w1 - w0;
  const int s0 = w0 + (len * wave) / 4, s1 = w0 + (len * (wave + 1)) / 4;
  const uint16_t *vbase = Vt + ((size_t)rb * nkb * 64 + lane) * 8;
  const uint16_t *xrow = x + (size_t)min(l32, B - 1) * n + q * 8;
  const bool xvalid = l32 < B;
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  u32x4 va[DEC_DEPTH], xa[DEC_DEPTH];
#pragma unroll
  for (int d = 0; d < DEC_DEPTH; ++d) {
    const int s = s0 + d;
    if (s < s1) {
      va[d] = *reinterpret_cast<const u32x4 *>(vbase + (size_t)s * 512);
      xa[d] = xvalid ? *reinterpret_cast<const u32x4 *>(xrow + (size_t)s * 16) : u32x4{0, 0, 0, 0};
    }
  }
  for (int sb = s0; sb < s1; sb += DEC_DEPTH) {
#pragma unroll
    for (int d = 0; d < DEC_DEPTH; ++d) {
      const int s = sb + d;
      if (s < s1) {
        const u32x4 cv = va[d], cx = xa[d];
        const int sn = s + DEC_DEPTH;
        if (sn < s1) {
          va[d] = *reinterpret_cast<const u32x4 *>(vbase + (size_t)sn * 512);
          xa[d] = xvalid ? *reinterpret_cast<const u32x4 *>(xrow + (size_t)sn * 16) : u32x4{0, 0, 0, 0};
        }
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(cv), dec_bf16x8(cx), acc, 0, 0, 0);
      }
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int e = 0; e < 16; ++e) red[wave - 1][e][lane] = acc[e];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] += red[0][e][lane] + red[1][e][lane] + red[2][e][lane];
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
                            const int32_t *__restrict__ pattern_id, uint16_t *__restrict__ zf) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= R * 4) return;   // R/16 * 64 pieces
  const int b = o & 31, q = (o >> 5) & 1, kb = o >> 6;
  const int r0 = kb * 16 + q * 8;
  const int g = r0 / gs;
  float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (seq_uses_group(subsets, stride, k, n_patterns, pattern_id, B, b, g)) {
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
                                                       const int32_t *__restrict__ subsets, int stride, int k,
                                                       int n_patterns, const int32_t *__restrict__ pattern_id,
                                                       uint16_t *__restrict__ y) {
  __shared__ float red[DY_THREADS / 64][16][64];
  __shared__ int32_t used[DEC_MAXG];
  __shared__ int32_t n_used_s;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, q = lane >> 5;
  const int cb = blockIdx.x, ncb = m / 32;
  // groups selected by at least one sequence, ascending
  if (wave == 0) {
    bool u = false;
    if (lane < G)
      for (int b = 0; b < B; ++b) u = u || seq_uses_group(subsets, stride, k, n_patterns, pattern_id, B, b, lane);
    const unsigned long long mask = __ballot(u);
    if (u) used[__popcll(mask & ((1ull << lane) - 1ull))] = lane;
    if (lane == 0) n_used_s = __popcll(mask);
  }
  __syncthreads();
  const int kpg = gs / 16;                 // reduction blocks per group
  const int total = n_used_s * kpg;        // selected reduction blocks
  constexpr int NW = DY_THREADS / 64;
  const int s0 = (total * wave) / NW, s1 = (total * (wave + 1)) / NW;
  const uint16_t *ubase = Ut + ((size_t)cb * 64 + lane) * 8;
  const uint16_t *zbase = zf + (size_t)lane * 8;
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  auto kb_of = [&](int s) { return used[s / kpg] * kpg + s % kpg; };
  u32x4 ua[DEC_DEPTH], za[DEC_DEPTH];
#pragma unroll
  for (int d = 0; d < DEC_DEPTH; ++d) {
    const int s = s0 + d;
    if (s < s1) {
      const int kb = kb_of(s);
      ua[d] = *reinterpret_cast<const u32x4 *>(ubase + (size_t)kb * ncb * 512);
      za[d] = *reinterpret_cast<const u32x4 *>(zbase + (size_t)kb * 512);
    }
  }
  for (int sb = s0; sb < s1; sb += DEC_DEPTH) {
#pragma unroll
    for (int d = 0; d < DEC_DEPTH; ++d) {
      const int s = sb + d;
      if (s < s1) {
        const u32x4 cu = ua[d], cz = za[d];
        const int sn = s + DEC_DEPTH;
        if (sn < s1) {
          const int kb = kb_of(sn);
          ua[d] = *reinterpret_cast<const u32x4 *>(ubase + (size_t)kb * ncb * 512);
          za[d] = *reinterpret_cast<const u32x4 *>(zbase + (size_t)kb * 512);
        }
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dec_bf16x8(cu), dec_bf16x8(cz), acc, 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) red[wave][e][lane] = acc[e];
  __syncthreads();
  // 16 x 64 sums over the NW wavefronts: thread (e, lane') for 1024 values, 2 per thread
  for (int i = threadIdx.x; i < 16 * 64; i += DY_THREADS) {
    const int e = i >> 6, ln = i & 63;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) s += red[w][e][ln];
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

static int decode_slices(int R) {
  int ks = (640 + R / 32 - 1) / (R / 32);
  if (ks < 1) ks = 1;
  if (ks > 16) ks = 16;
  return ks;
}

size_t decode_workspace_bytes(const parse_layer *L) {
  const int KS = decode_slices(L->R);
  return round_up((size_t)KS * 32 * L->R * sizeof(float), 256) + round_up((size_t)L->R * 32 * sizeof(uint16_t), 256);
}

int forward_decode_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *x, int B,
                        const int32_t *pattern_id, uint16_t *y, void *workspace, hipStream_t s) {
  const int gs = L->R / L->G;
  const int KS = decode_slices(L->R);
  float *zp = reinterpret_cast<float *>(workspace);
  uint16_t *zf = reinterpret_cast<uint16_t *>((char *)workspace + round_up((size_t)KS * 32 * L->R * sizeof(float), 256));
  hipLaunchKernelGGL(decode_z, dim3(L->R / 32, KS), dim3(DZ_THREADS), 0, s, (const uint16_t *)L->Vt, x, B, L->n, L->R,
                     gs, pt->subsets, pt->subset_stride, pt->k, pt->n_patterns, pattern_id, KS, zp);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(decode_zfin, dim3((L->R * 4 + 255) / 256), dim3(256), 0, s, zp, KS, B, L->R, gs, pt->subsets,
                     pt->subset_stride, pt->k, pt->n_patterns, pattern_id, zf);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(decode_y, dim3(L->m / 32), dim3(DY_THREADS), 0, s, (const uint16_t *)L->Ut, zf, B, L->m, L->R,
                     L->G, gs, pt->subsets, pt->subset_stride, pt->k, pt->n_patterns, pattern_id, y);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // namespace parse
