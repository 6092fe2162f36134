// a6 for fp32 layers (correctness configuration): Y = (X Vt_S^T) Ut_S with plain fp32 FMA tiles.
// Two launches of one LDS-tiled kernel; the r_S-wide intermediate goes through the workspace.
// Each 64-row block of the flat token axis is cut into the segments that belong to one prompt, and a
// segment uses the packed factors of that prompt's pattern.
#include "common.hpp"

namespace parse {

constexpr int TM = 64, TN = 64, TK = 16;

// C[rows][N] = A[rows][K] * op(B_p).  B_NT: B_p is [N][K] (Vt_S);  else B_p is [K][N] (Ut_S).
template <bool B_NT>
__global__ __launch_bounds__(256) void sgemm_segments(const float *__restrict__ A, const float *__restrict__ Bbase,
                                                      size_t pattern_stride, int n_patterns, int rows, int N, int K,
                                                      const int32_t *__restrict__ tok_offsets,
                                                      const int32_t *__restrict__ pattern_id, int P,
                                                      float *__restrict__ C) {
  __shared__ float As[TK][TM + 1];
  __shared__ float Bs[TK][TN + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int row0 = blockIdx.x * TM, col0 = blockIdx.y * TN;
  const int row_end = min(row0 + TM, rows);
  int seg_lo = row0;
  while (seg_lo < row_end) {
    const int p = prompt_of_row(tok_offsets, P, seg_lo);
    int seg_hi = (p + 1 < P) ? tok_offsets[p + 1] : rows;   // the last prompt owns every remaining row
    seg_hi = min(max(seg_hi, seg_lo + 1), row_end);
    const int pid = pattern_id[p];
    const bool valid = pid >= 0 && pid < n_patterns;
    const float *B = Bbase + (valid ? (size_t)pid * pattern_stride : 0);
    float acc[4][4] = {};
    if (valid) {
      for (int k0 = 0; k0 < K; k0 += TK) {
        // A tile: 64 rows x 16 k; thread loads 4 elements
        for (int i = threadIdx.x; i < TM * TK; i += 256) {
          const int r = i / TK, kk = i % TK;
          const int gr = min(row0 + r, rows - 1), gk = k0 + kk;
          As[kk][r] = (gk < K) ? A[(size_t)gr * K + gk] : 0.f;
        }
        for (int i = threadIdx.x; i < TN * TK; i += 256) {
          int c, kk;
          if (B_NT) { c = i / TK; kk = i % TK; } else { kk = i / TN; c = i % TN; }
          const int gc = col0 + c, gk = k0 + kk;
          float v = 0.f;
          if (gc < N && gk < K) v = B_NT ? B[(size_t)gc * K + gk] : B[(size_t)gk * N + gc];
          Bs[kk][c] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
          float a[4], b[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = row0 + ty * 4 + i;
      if (r < seg_lo || r >= seg_hi) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = col0 + tx * 4 + j;
        if (c < N) C[(size_t)r * N + c] = acc[i][j];
      }
    }
    seg_lo = seg_hi;
  }
}

int forward_f32(const parse_layer *L, const parse_patterns *pt, const float *X, int rows, const int32_t *tok_offsets,
                const int32_t *pattern_id, int P, float *Y, void *workspace, hipStream_t s) {
  const int gs = L->R / L->G, rS = pt->k * gs;
  float *Z = reinterpret_cast<float *>(workspace);
  dim3 g1((rows + TM - 1) / TM, (rS + TN - 1) / TN);
  hipLaunchKernelGGL(sgemm_segments<true>, g1, dim3(256), 0, s, X, (const float *)pt->Vt_S, (size_t)rS * L->n,
                     pt->n_patterns, rows, rS, L->n, tok_offsets, pattern_id, P, Z);
  PARSE_LAUNCH_CHECK();
  dim3 g2((rows + TM - 1) / TM, (L->m + TN - 1) / TN);
  hipLaunchKernelGGL(sgemm_segments<false>, g2, dim3(256), 0, s, Z, (const float *)pt->Ut_S, (size_t)rS * L->m,
                     pt->n_patterns, rows, L->m, rS, tok_offsets, pattern_id, P, Y);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // namespace parse
