// Router training step (Sec. 4.2, "Calibration-Decoupled Router Training"): the low-rank factors stay fixed, the
// router matrix is trained against the dense model's output with the reconstruction loss of Eq. 6; the forward
// pass uses the hard top-k mask (Eq. 7), the backward pass the K-normalised sigmoid mask (Eq. 8-9, straight
// through).  This file computes loss and gradient for one batch of prompts, groups as experts, one embedding per
// prompt, given the routed output Y_hat (parse_lowrank_forward) and the dense output Y_dense:
//   residual       g = 2 (y_hat - y_dense) per token (bf16), squared-error sum per token row
//   two products   Z = X V^T and Tm = g U over ALL stored ranks (the first-product matrix kernel, twice)
//   mask_grad      dL/dm[p][group] = sum over the prompt's tokens and the group's ranks of Z * Tm
//   router_grad    dL/ds_j = k a'_j (dL/dm_j / A - B / A^2) with a = sigmoid(s / tau), a' = a (1 - a) / tau,
//                  A = sum a + eps, B = sum_g dL/dm_g a_g  (the Jacobian of Eq. 9 applied in closed form), then
//                  dL/dWr[j][:] = sum_p dL/ds_j(p) e_p, prompts added in order.
// No atomics: same inputs, same bits.
#include "common.hpp"

namespace parse {

int tokens_times_factor_bf16(const uint16_t *Tk, const uint16_t *F, uint16_t *O, int rows, int K, int M,
                             const int32_t *one_offsets, const int32_t *zero_id, hipStream_t s);

// grid rows, block 256.  Block 0 also writes the helper index arrays of the two products.
__global__ __launch_bounds__(256) void train_residual(const uint16_t *__restrict__ Yh, const uint16_t *__restrict__ Yd,
                                                      int rows, int m, uint16_t *__restrict__ g,
                                                      float *__restrict__ rowloss, int32_t *__restrict__ helper) {
  __shared__ float red[256];
  const int t = blockIdx.x;
  if (t == 0 && threadIdx.x == 0) { helper[0] = 0; helper[1] = rows; helper[2] = 0; }
  float acc = 0.f;
  for (int c = threadIdx.x * 8; c < m; c += 256 * 8) {
    const u32x4 a = *reinterpret_cast<const u32x4 *>(Yh + (size_t)t * m + c);
    const u32x4 b = *reinterpret_cast<const u32x4 *>(Yd + (size_t)t * m + c);
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float d0 = __uint_as_float(a[i] << 16) - __uint_as_float(b[i] << 16);
      const float d1 = __uint_as_float(a[i] & 0xFFFF0000u) - __uint_as_float(b[i] & 0xFFFF0000u);
      acc += d0 * d0 + d1 * d1;
      w[i] = pack_bf16x2(2.f * d0, 2.f * d1);
    }
    *reinterpret_cast<u32x4 *>(g + (size_t)t * m + c) = w;
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) rowloss[t] = red[0];
}

// grid (G, P), block 256: lane handles rank (tid % gs_lanes) ... of the group for every (256 / gs_lanes)-th token.
__global__ __launch_bounds__(256) void train_mask_grad(const uint16_t *__restrict__ Z, const uint16_t *__restrict__ Tm,
                                                       int rows, int R, int gs, const int32_t *__restrict__ tok_offsets,
                                                       float *__restrict__ dm, int G) {
  __shared__ float red[256];
  const int g = blockIdx.x, p = blockIdx.y;
  int a = tok_offsets[p], b = tok_offsets[p + 1];
  a = a < 0 ? 0 : (a > rows ? rows : a);
  b = b < a ? a : (b > rows ? rows : b);
  const int pieces = gs / 8;                      // 16-byte pieces per token row of the group
  float acc = 0.f;
  for (long long w = threadIdx.x; w < (long long)(b - a) * pieces; w += 256) {
    const int t = a + (int)(w / pieces), c = g * gs + (int)(w % pieces) * 8;
    const u32x4 zv = *reinterpret_cast<const u32x4 *>(Z + (size_t)t * R + c);
    const u32x4 tv = *reinterpret_cast<const u32x4 *>(Tm + (size_t)t * R + c);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      acc += __uint_as_float(zv[i] << 16) * __uint_as_float(tv[i] << 16) +
             __uint_as_float(zv[i] & 0xFFFF0000u) * __uint_as_float(tv[i] & 0xFFFF0000u);
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) dm[(size_t)p * G + g] = red[0];
}

constexpr int TR_MAX_PG = 8192;   // P * G entries of dL/ds a workgroup keeps in LDS

// grid ceil(d / 256), block 256.  Every workgroup first works out dL/ds[p][j] for the whole batch (LDS), then its
// 256 columns of the gradient; workgroup 0 also adds up the per-prompt losses.
__global__ __launch_bounds__(256) void train_router_grad(const float *__restrict__ dm, const float *__restrict__ scores,
                                                         const float *__restrict__ emb, int P, int G, int d, int k,
                                                         float inv_tau, float eps, const float *__restrict__ rowloss,
                                                         const int32_t *__restrict__ tok_offsets, int rows,
                                                         float *__restrict__ loss_out, float *__restrict__ grad) {
  __shared__ float ds[TR_MAX_PG];
  for (int p = threadIdx.x; p < P; p += 256) {
    float A = eps, B = 0.f;
    for (int g = 0; g < G; ++g) {
      const float sg = 1.f / (1.f + expf(-scores[(size_t)p * G + g] * inv_tau));
      A += sg;
      B += dm[(size_t)p * G + g] * sg;
    }
    for (int j = 0; j < G; ++j) {
      const float sg = 1.f / (1.f + expf(-scores[(size_t)p * G + j] * inv_tau));
      const float dsg = sg * (1.f - sg) * inv_tau;
      ds[p * G + j] = (float)k * dsg * (dm[(size_t)p * G + j] / A - B / (A * A));
    }
    if (blockIdx.x == 0 && loss_out) {
      int a = tok_offsets[p], b = tok_offsets[p + 1];
      a = a < 0 ? 0 : (a > rows ? rows : a);
      b = b < a ? a : (b > rows ? rows : b);
      float l = 0.f;
      for (int t = a; t < b; ++t) l += rowloss[t];
      loss_out[p] = l;
    }
  }
  __syncthreads();
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d) return;
  for (int j = 0; j < G; ++j) {
    float acc = 0.f;
    for (int p = 0; p < P; ++p) acc += ds[p * G + j] * emb[(size_t)p * d + c];
    grad[(size_t)j * d + c] = acc;
  }
}

}  // namespace parse

using namespace parse;

extern "C" {

size_t parse_router_grad_workspace_bytes(const parse_layer *L, int32_t rows, int32_t P) {
  if (!L || rows <= 0 || P <= 0 || L->R <= 0 || L->G <= 0 || L->m <= 0) return 0;
  return round_up((size_t)rows * L->m * 2, 256) + 2 * round_up((size_t)rows * L->R * 2, 256) +
         round_up((size_t)rows * sizeof(float), 256) + round_up((size_t)P * L->G * sizeof(float), 256) + 256;
}

int parse_router_grad(const parse_layer *L, const void *Ut_rankmajor, const void *X, int32_t rows,
                      const int32_t *tok_offsets, int32_t P, const void *Y_hat, const void *Y_dense,
                      const float *emb, const float *scores, int32_t d, int32_t k, float temperature, float eps,
                      float *loss_out, float *grad_Wr, void *workspace, size_t workspace_bytes,
                      parse_stream stream) {
  int st = check_layer(L);
  if (st != PARSE_OK) return st;
  if (!Ut_rankmajor || !X || !tok_offsets || !Y_hat || !Y_dense || !emb || !scores || !grad_Wr) return PARSE_EINVAL;
  if (rows <= 0 || P <= 0 || d <= 0 || k <= 0 || !(temperature > 0.f) || eps < 0.f) return PARSE_EINVAL;
  if (L->dtype != PARSE_BF16 || L->layout != PARSE_MFMA16) return PARSE_ELAYOUT;
  const int gs = L->R / L->G;
  if (k > L->G || L->G > 64 || P > rows || (long long)P * L->G > TR_MAX_PG) return PARSE_ESHAPE;
  if (L->n % 128 != 0 || L->m % 128 != 0 || L->R % 32 != 0 || gs % 8 != 0) return PARSE_ESHAPE;
  if (!aligned16(Ut_rankmajor) || !aligned16(X) || !aligned16(Y_hat) || !aligned16(Y_dense) || !aligned16(emb))
    return PARSE_EALIGN;
  if (!workspace || workspace_bytes < parse_router_grad_workspace_bytes(L, rows, P)) return PARSE_EWORKSPACE;
  if (!aligned16(workspace)) return PARSE_EALIGN;
  hipStream_t s = (hipStream_t)stream;
  char *ws = reinterpret_cast<char *>(workspace);
  uint16_t *g = reinterpret_cast<uint16_t *>(ws);            ws += round_up((size_t)rows * L->m * 2, 256);
  uint16_t *Z = reinterpret_cast<uint16_t *>(ws);            ws += round_up((size_t)rows * L->R * 2, 256);
  uint16_t *Tm = reinterpret_cast<uint16_t *>(ws);           ws += round_up((size_t)rows * L->R * 2, 256);
  float *rowloss = reinterpret_cast<float *>(ws);            ws += round_up((size_t)rows * sizeof(float), 256);
  float *dm = reinterpret_cast<float *>(ws);                 ws += round_up((size_t)P * L->G * sizeof(float), 256);
  int32_t *helper = reinterpret_cast<int32_t *>(ws);         // {0, rows} offsets of one all-rows prompt, {0} its id
  hipLaunchKernelGGL(train_residual, dim3(rows), dim3(256), 0, s, (const uint16_t *)Y_hat, (const uint16_t *)Y_dense,
                     rows, L->m, g, rowloss, helper);
  PARSE_LAUNCH_CHECK();
  st = tokens_times_factor_bf16((const uint16_t *)X, (const uint16_t *)L->Vt, Z, rows, L->n, L->R, helper, helper + 2, s);
  if (st != PARSE_OK) return st;
  st = tokens_times_factor_bf16(g, (const uint16_t *)Ut_rankmajor, Tm, rows, L->m, L->R, helper, helper + 2, s);
  if (st != PARSE_OK) return st;
  hipLaunchKernelGGL(train_mask_grad, dim3(L->G, P), dim3(256), 0, s, Z, Tm, rows, L->R, gs, tok_offsets, dm, L->G);
  PARSE_LAUNCH_CHECK();
  hipLaunchKernelGGL(train_router_grad, dim3((d + 255) / 256), dim3(256), 0, s, dm, scores, emb, P, L->G, d, k,
                     1.0f / temperature, eps, rowloss, tok_offsets, rows, loss_out, grad_Wr);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // extern "C"
