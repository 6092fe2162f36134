// parse_lowrank_forward: argument checks and dispatch to the fp32 / bf16 prefill kernels and the decode kernels.
#include "prefill_common.hpp"

namespace parse {
int forward_f32(const parse_layer *L, const parse_patterns *pt, const float *X, int rows, const int32_t *tok_offsets,
                const int32_t *pattern_id, int P, float *Y, void *workspace, hipStream_t s);
int forward_prefill_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *X, int rows,
                         const int32_t *tok_offsets, const int32_t *pattern_id, int P, uint16_t *Y, void *workspace,
                         size_t workspace_bytes, hipStream_t s);
size_t prefill_split_workspace_bytes(int rows, int rS);
bool prefill_split_supported(int n, int rS);
int forward_prefill_split_multi_bf16(const PfArgs *p, int n_layers, uint16_t *const *Z, int avg_prompt_rows, hipStream_t s);
size_t prefill_plan_bytes(int rows, int P, int n_patterns);
int prefill_plan_capacity(int rows, int P, int n_patterns);
bool prefill_plan_supported(int P, int n_patterns);
int build_prefill_plan(const int32_t *tok_offsets, const int32_t *pattern_id, int P, int rows, int n_patterns,
                       int32_t *plan, hipStream_t s);
size_t prefill_planned_z_bytes(int cap_tiles, int rS, int ks);
int prefill_planned_split(int rows, int n);
bool prefill_planned_supported(int n, int m, int rS);
int forward_prefill_planned_multi_bf16(const PfArgs *p, int n_layers, const int32_t *plan, int cap, uint16_t *const *Z,
                                       int avg_prompt_rows, hipStream_t s);
int forward_prefill_planned_bf16(const PfArgs &p, const int32_t *plan, int cap, uint16_t *Z, int avg_prompt_rows,
                                 hipStream_t s);
size_t prefill_lds_bytes(int BM, int rS);
size_t decode_workspace_bytes(const parse_layer *L);
size_t decode_plan_bytes(int n_layers);
size_t decode_z_bytes(const parse_layer *layers, int n_layers);
bool decode_supported(const parse_layer *L);
int build_decode_plan(const parse_layer *layers, const parse_patterns *pts, int n_layers, const int32_t *pattern_id,
                      int B, int32_t *plan, hipStream_t s);
int forward_decode_planned_bf16(const parse_layer *layers, int n_layers, const uint16_t *x, int B, int32_t *plan,
                                uint16_t *const *Y, void *workspace, hipStream_t s);
int forward_decode_multi_bf16(const parse_layer *layers, const parse_patterns *pts, int n_layers, const uint16_t *x,
                              int B, const int32_t *pattern_id, uint16_t *const *Y, void *workspace, hipStream_t s);
int forward_decode_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *x, int B,
                        const int32_t *pattern_id, uint16_t *y, void *workspace, hipStream_t s);
}  // namespace parse

using namespace parse;

extern "C" {

// workspace of the planned schedule inside parse_lowrank_forward: the intermediate, then the plan
static size_t planned_total_bytes(const parse_layer *L, int rows, int P, int k, int n_patterns) {
  const int rS = k * (L->R / L->G);
  return prefill_planned_z_bytes(prefill_plan_capacity(rows, P, n_patterns), rS, prefill_planned_split(rows, L->n)) +
         prefill_plan_bytes(rows, P, n_patterns);
}

size_t parse_lowrank_workspace_bytes(int32_t mode, const parse_layer *L, int32_t rows, int32_t k, int32_t P,
                                     int32_t n_patterns) {
  if (!L || rows <= 0 || k <= 0 || L->G <= 0 || L->R <= 0) return 0;
  if (mode == PARSE_DECODE) return decode_workspace_bytes(L);
  if (L->dtype == PARSE_F32) return round_up((size_t)rows * k * (L->R / L->G) * sizeof(float), 256);
  const int rS = k * (L->R / L->G);
  size_t need = prefill_split_workspace_bytes(rows, rS);
  if (P > 0 && n_patterns > 0 && P <= rows && prefill_plan_supported(P, n_patterns) &&
      prefill_planned_supported(L->n, L->m, rS)) {
    const size_t planned = planned_total_bytes(L, rows, P, k, n_patterns);
    if (planned > need) need = planned;
  }
  return need;
}

size_t parse_lowrank_prefill_planned_workspace_bytes(const parse_layer *L, int32_t rows, int32_t P, int32_t k,
                                                     int32_t n_patterns) {
  if (!L || rows <= 0 || k <= 0 || P <= 0 || n_patterns <= 0 || L->G <= 0 || L->R <= 0) return 0;
  const int rS = k * (L->R / L->G);
  return prefill_planned_z_bytes(prefill_plan_capacity(rows, P, n_patterns), rS, prefill_planned_split(rows, L->n));
}

int parse_lowrank_prefill_planned(const parse_layer *L, const parse_patterns *pt, const void *X, int32_t rows,
                                  const int32_t *tok_offsets, const int32_t *pattern_id, int32_t P, const void *plan,
                                  void *Y, void *workspace, size_t workspace_bytes, parse_stream stream) {
  int st = check_layer(L);
  if (st != PARSE_OK) return st;
  if (!pt || !X || !Y || !plan || !tok_offsets || !pattern_id || !pt->Vt_S || !pt->Ut_S) return PARSE_EINVAL;
  if (rows <= 0 || P <= 0 || pt->n_patterns <= 0 || pt->k <= 0) return PARSE_EINVAL;
  if (L->dtype != PARSE_BF16 || L->layout != PARSE_MFMA16) return PARSE_ELAYOUT;
  if (pt->n_shared < 0) return PARSE_EINVAL;
  const int rS = pt->k * (L->R / L->G);
  if (pt->n_shared > 0) {   // shared head: whole 32-rank blocks, stored once
    if (!pt->Vt_shared || !pt->Ut_shared) return PARSE_EINVAL;
    if (pt->n_shared >= pt->k || (pt->n_shared * (L->R / L->G)) % 32 != 0) return PARSE_ESHAPE;
    if (!aligned16(pt->Vt_shared) || !aligned16(pt->Ut_shared)) return PARSE_EALIGN;
  }
  if (pt->k > L->G || P > rows || !prefill_plan_supported(P, pt->n_patterns) ||
      !prefill_planned_supported(L->n, L->m, rS)) return PARSE_ESHAPE;
  if (!aligned16(X) || !aligned16(Y) || !aligned16(plan) || !aligned16(pt->Vt_S) || !aligned16(pt->Ut_S)) return PARSE_EALIGN;
  const int cap = prefill_plan_capacity(rows, P, pt->n_patterns);
  if (!workspace || workspace_bytes < prefill_planned_z_bytes(cap, rS, prefill_planned_split(rows, L->n)))
    return PARSE_EWORKSPACE;
  if (!aligned16(workspace)) return PARSE_EALIGN;
  PfArgs a{(const uint16_t *)X, (const uint16_t *)pt->Vt_S, (const uint16_t *)pt->Ut_S, (uint16_t *)Y, tok_offsets, pattern_id,
           pt->n_patterns, rows, L->n, L->m, rS, P};
  if (pt->n_shared > 0) {
    a.Vt_sh = (const uint16_t *)pt->Vt_shared;
    a.Ut_sh = (const uint16_t *)pt->Ut_shared;
    a.sh_ranks = pt->n_shared * (L->R / L->G);
  }
  return forward_prefill_planned_bf16(a, (const int32_t *)plan, cap, (uint16_t *)workspace, rows / P, (hipStream_t)stream);
}

int parse_lowrank_forward(int32_t mode, const parse_layer *L, const parse_patterns *pt, const void *X, int32_t rows,
                          const int32_t *tok_offsets, const int32_t *pattern_id, int32_t P, void *Y, void *workspace,
                          size_t workspace_bytes, parse_stream stream) {
  if (mode != PARSE_PREFILL && mode != PARSE_DECODE) return PARSE_EINVAL;
  int st = check_layer(L);
  if (st != PARSE_OK) return st;
  if (!pt || !X || !Y || !pattern_id) return PARSE_EINVAL;
  if (rows <= 0 || P <= 0 || pt->n_patterns <= 0 || pt->k <= 0) return PARSE_EINVAL;
  if (pt->k > L->G || P > rows) return PARSE_ESHAPE;
  if (!aligned16(X) || !aligned16(Y)) return PARSE_EALIGN;
  if (mode == PARSE_DECODE && (L->dtype != PARSE_BF16 || L->layout != PARSE_MFMA16)) return PARSE_ELAYOUT;
  const size_t need = parse_lowrank_workspace_bytes(mode, L, rows, pt->k, 0, 0);   // the smallest workspace any schedule takes
  // bf16 prefill may run without a workspace (fused kernel only); every other mode needs the queried size
  const bool optional_ws = mode == PARSE_PREFILL && L->dtype == PARSE_BF16 && workspace == nullptr;
  if (!optional_ws && need > 0 && (!workspace || workspace_bytes < need)) return PARSE_EWORKSPACE;
  if (workspace && !aligned16(workspace)) return PARSE_EALIGN;
  hipStream_t s = (hipStream_t)stream;
  const int gs = L->R / L->G, rS = pt->k * gs;

  if (mode == PARSE_DECODE) {
    if (!pt->subsets) return PARSE_EINVAL;
    if (rows != P || L->G > 64 || pt->subset_stride < pt->k) return PARSE_ESHAPE;
    // panels of 32 sequences (the matrix instruction's N side); every panel has its own masks and streams the groups
    // its own sequences selected
    for (int r0 = 0; r0 < rows; r0 += 32) {
      const int nb = rows - r0 < 32 ? rows - r0 : 32;
      st = forward_decode_bf16(L, pt, (const uint16_t *)X + (size_t)r0 * L->n, nb, pattern_id + r0,
                               (uint16_t *)Y + (size_t)r0 * L->m, workspace, s);
      if (st != PARSE_OK) return st;
    }
    return PARSE_OK;
  }

  if (!tok_offsets || !pt->Vt_S || !pt->Ut_S) return PARSE_EINVAL;
  if (!aligned16(pt->Vt_S) || !aligned16(pt->Ut_S)) return PARSE_EALIGN;
  if (pt->n_shared < 0) return PARSE_EINVAL;
  if (pt->n_shared > 0) {   // shared head: bf16 operand-order layers, two-launch schedule
    if (L->dtype != PARSE_BF16 || L->layout != PARSE_MFMA16) return PARSE_ELAYOUT;
    if (!pt->Vt_shared || !pt->Ut_shared) return PARSE_EINVAL;
    if (pt->n_shared >= pt->k) return PARSE_ESHAPE;
    if (!aligned16(pt->Vt_shared) || !aligned16(pt->Ut_shared)) return PARSE_EALIGN;
  }
  if (L->dtype == PARSE_F32) {
    if (L->layout != PARSE_ROWMAJOR) return PARSE_ELAYOUT;
    return forward_f32(L, pt, (const float *)X, rows, tok_offsets, pattern_id, P, (float *)Y, workspace, s);
  }
  if (L->layout != PARSE_MFMA16) return PARSE_ELAYOUT;
  if (rS % 32 != 0) return PARSE_ESHAPE;
  if (prefill_lds_bytes(32, rS) > 160 * 1024) return PARSE_ESHAPE;
  return forward_prefill_bf16(L, pt, (const uint16_t *)X, rows, tok_offsets, pattern_id, P, (uint16_t *)Y, workspace,
                              workspace_bytes, s);
}

size_t parse_lowrank_decode_multi_workspace_bytes(const parse_layer *layers, int32_t n_layers) {
  if (!layers || n_layers < 1 || n_layers > 4) return 0;
  for (int l = 0; l < n_layers; ++l)
    if (layers[l].G <= 0 || layers[l].R <= 0) return 0;
  return decode_z_bytes(layers, n_layers) + decode_plan_bytes(n_layers);   // the call builds its plan behind the intermediates
}

int parse_lowrank_decode_multi(const parse_layer *layers, const parse_patterns *patterns, int32_t n_layers,
                               const void *X, int32_t rows, const int32_t *pattern_id, void *const *Y,
                               void *workspace, size_t workspace_bytes, parse_stream stream) {
  if (!layers || !patterns || !X || !pattern_id || !Y) return PARSE_EINVAL;
  if (n_layers < 1 || rows <= 0) return PARSE_EINVAL;
  if (n_layers > 4) return PARSE_ESHAPE;
  if (!aligned16(X)) return PARSE_EALIGN;
  for (int l = 0; l < n_layers; ++l) {
    const parse_layer *L = &layers[l];
    const parse_patterns *pt = &patterns[l];
    int st = check_layer(L);
    if (st != PARSE_OK) return st;
    if (L->dtype != PARSE_BF16 || L->layout != PARSE_MFMA16) return PARSE_ELAYOUT;
    if (!Y[l] || !pt->subsets) return PARSE_EINVAL;
    if (pt->n_patterns <= 0 || pt->k <= 0) return PARSE_EINVAL;
    if (pt->k > L->G || L->G > 64 || pt->subset_stride < pt->k || L->n != layers[0].n) return PARSE_ESHAPE;
    if (!aligned16(Y[l])) return PARSE_EALIGN;
  }
  const size_t need = parse_lowrank_decode_multi_workspace_bytes(layers, n_layers);
  if (!workspace || workspace_bytes < need) return PARSE_EWORKSPACE;
  if (!aligned16(workspace)) return PARSE_EALIGN;
  // panels of 32 sequences, as in parse_lowrank_forward(PARSE_DECODE)
  for (int r0 = 0; r0 < rows; r0 += 32) {
    const int nb = rows - r0 < 32 ? rows - r0 : 32;
    uint16_t *Yp[4] = {nullptr, nullptr, nullptr, nullptr};
    for (int l = 0; l < n_layers; ++l) Yp[l] = (uint16_t *)Y[l] + (size_t)r0 * layers[l].m;
    const int st = forward_decode_multi_bf16(layers, patterns, n_layers, (const uint16_t *)X + (size_t)r0 * layers[0].n, nb,
                                             pattern_id + r0, Yp, workspace, (hipStream_t)stream);
    if (st != PARSE_OK) return st;
  }
  return PARSE_OK;
}

// checks shared by the decode entry points that take several layers
static int check_decode_layers(const parse_layer *layers, int32_t n_layers) {
  if (!layers || n_layers < 1) return PARSE_EINVAL;
  if (n_layers > 4) return PARSE_ESHAPE;
  for (int l = 0; l < n_layers; ++l) {
    int st = check_layer(&layers[l]);
    if (st != PARSE_OK) return st;
    if (layers[l].dtype != PARSE_BF16 || layers[l].layout != PARSE_MFMA16) return PARSE_ELAYOUT;
    if (layers[l].G > 64 || layers[l].n != layers[0].n || !decode_supported(&layers[l])) return PARSE_ESHAPE;
  }
  return PARSE_OK;
}

size_t parse_decode_plan_bytes(int32_t n_layers) {
  if (n_layers < 1 || n_layers > 4) return 0;
  return decode_plan_bytes(n_layers);
}

int parse_decode_plan(const parse_layer *layers, const parse_patterns *patterns, int32_t n_layers,
                      const int32_t *pattern_id, int32_t rows, void *plan, size_t plan_bytes, parse_stream stream) {
  if (!patterns || !pattern_id || !plan) return PARSE_EINVAL;
  int st = check_decode_layers(layers, n_layers);
  if (st != PARSE_OK) return st;
  if (rows <= 0) return PARSE_EINVAL;
  if (rows > 32) return PARSE_ESHAPE;
  for (int l = 0; l < n_layers; ++l) {
    if (!patterns[l].subsets || patterns[l].n_patterns <= 0 || patterns[l].k <= 0) return PARSE_EINVAL;
    if (patterns[l].k > layers[l].G || patterns[l].subset_stride < patterns[l].k) return PARSE_ESHAPE;
  }
  if (!aligned16(plan)) return PARSE_EALIGN;
  if (plan_bytes < decode_plan_bytes(n_layers)) return PARSE_EWORKSPACE;
  return build_decode_plan(layers, patterns, n_layers, pattern_id, rows, (int32_t *)plan, (hipStream_t)stream);
}

size_t parse_lowrank_decode_planned_workspace_bytes(const parse_layer *layers, int32_t n_layers) {
  if (!layers || n_layers < 1 || n_layers > 4) return 0;
  for (int l = 0; l < n_layers; ++l)
    if (layers[l].G <= 0 || layers[l].R <= 0) return 0;
  return decode_z_bytes(layers, n_layers);
}

int parse_lowrank_decode_planned(const parse_layer *layers, int32_t n_layers, const void *X, int32_t rows,
                                 void *plan, void *const *Y, void *workspace, size_t workspace_bytes,
                                 parse_stream stream) {
  if (!X || !plan || !Y) return PARSE_EINVAL;
  int st = check_decode_layers(layers, n_layers);
  if (st != PARSE_OK) return st;
  if (rows <= 0) return PARSE_EINVAL;
  if (rows > 32) return PARSE_ESHAPE;
  if (!aligned16(X) || !aligned16(plan)) return PARSE_EALIGN;
  for (int l = 0; l < n_layers; ++l) {
    if (!Y[l]) return PARSE_EINVAL;
    if (!aligned16(Y[l])) return PARSE_EALIGN;
  }
  if (!workspace || workspace_bytes < decode_z_bytes(layers, n_layers)) return PARSE_EWORKSPACE;
  if (!aligned16(workspace)) return PARSE_EALIGN;
  return forward_decode_planned_bf16(layers, n_layers, (const uint16_t *)X, rows, (int32_t *)plan,
                                     (uint16_t *const *)Y, workspace, (hipStream_t)stream);
}

// workspace of the planned schedule for several layers: every layer's padded intermediate, then the plan.  The plan's
// capacity is bounded without knowing the number of prompts (at most n_patterns + 1 pattern buckets).
static bool multi_planned_shapes(const parse_layer *layers, const parse_patterns *patterns, int n_layers) {
  for (int l = 0; l < n_layers; ++l) {
    const parse_layer *L = &layers[l];
    const parse_patterns *pt = &patterns[l];
    if (L->G <= 0 || L->R % L->G != 0) return false;
    const int gs = L->R / L->G;
    if (pt->n_patterns != patterns[0].n_patterns || pt->n_patterns > 2048) return false;
    if (!prefill_planned_supported(L->n, L->m, pt->k * gs)) return false;
    if (pt->n_shared < 0 || (pt->n_shared * gs) % 32 != 0) return false;
  }
  return true;
}
static size_t multi_planned_bytes(const parse_layer *layers, const parse_patterns *patterns, int n_layers, int rows, int P) {
  const int cap = prefill_plan_capacity(rows, P, patterns[0].n_patterns);
  size_t total = prefill_plan_bytes(rows, P, patterns[0].n_patterns);
  const int ks = prefill_planned_split(rows, layers[0].n);
  for (int l = 0; l < n_layers; ++l) total += prefill_planned_z_bytes(cap, patterns[l].k * (layers[l].R / layers[l].G), ks);
  return total;
}

size_t parse_lowrank_prefill_multi_workspace_bytes(const parse_layer *layers, const parse_patterns *patterns,
                                                   int32_t n_layers, int32_t rows) {
  if (!layers || !patterns || n_layers < 1 || n_layers > 4 || rows <= 0) return 0;
  size_t total = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (layers[l].G <= 0 || layers[l].R <= 0 || patterns[l].k <= 0) return 0;
    total += prefill_split_workspace_bytes(rows, patterns[l].k * (layers[l].R / layers[l].G));
  }
  if (multi_planned_shapes(layers, patterns, n_layers)) {
    const int p_ub = rows < 2048 ? rows : 2048;          // the plan takes at most 2048 prompts
    const size_t planned = multi_planned_bytes(layers, patterns, n_layers, rows, p_ub);
    if (planned > total) total = planned;
  }
  return total;
}

int parse_lowrank_prefill_multi(const parse_layer *layers, const parse_patterns *patterns, int32_t n_layers,
                                const void *X, int32_t rows, const int32_t *tok_offsets, const int32_t *pattern_id,
                                int32_t P, void *const *Y, void *workspace, size_t workspace_bytes,
                                parse_stream stream) {
  if (!layers || !patterns || !X || !tok_offsets || !pattern_id || !Y) return PARSE_EINVAL;
  if (n_layers < 1 || rows <= 0 || P <= 0) return PARSE_EINVAL;
  if (n_layers > 4 || P > rows) return PARSE_ESHAPE;
  if (!aligned16(X)) return PARSE_EALIGN;
  PfArgs args[4];
  bool tiles_ok = true;
  for (int l = 0; l < n_layers; ++l) {
    const parse_layer *L = &layers[l];
    const parse_patterns *pt = &patterns[l];
    int st = check_layer(L);
    if (st != PARSE_OK) return st;
    if (L->dtype != PARSE_BF16 || L->layout != PARSE_MFMA16) return PARSE_ELAYOUT;
    if (!Y[l] || !pt->Vt_S || !pt->Ut_S) return PARSE_EINVAL;
    if (pt->n_patterns <= 0 || pt->k <= 0) return PARSE_EINVAL;
    const int rS = pt->k * (L->R / L->G);
    if (pt->k > L->G || L->n != layers[0].n) return PARSE_ESHAPE;
    tiles_ok = tiles_ok && prefill_split_supported(L->n, rS);
    if (!aligned16(Y[l]) || !aligned16(pt->Vt_S) || !aligned16(pt->Ut_S)) return PARSE_EALIGN;
    args[l] = PfArgs{(const uint16_t *)X, (const uint16_t *)pt->Vt_S, (const uint16_t *)pt->Ut_S, (uint16_t *)Y[l],
                     tok_offsets, pattern_id, pt->n_patterns, rows, L->n, L->m, rS, P};
    if (pt->n_shared < 0) return PARSE_EINVAL;
    if (pt->n_shared > 0) {
      if (!pt->Vt_shared || !pt->Ut_shared) return PARSE_EINVAL;
      if (pt->n_shared >= pt->k) return PARSE_ESHAPE;
      if (!aligned16(pt->Vt_shared) || !aligned16(pt->Ut_shared)) return PARSE_EALIGN;
      args[l].Vt_sh = (const uint16_t *)pt->Vt_shared;
      args[l].Ut_sh = (const uint16_t *)pt->Ut_shared;
      args[l].sh_ranks = pt->n_shared * (L->R / L->G);
    }
  }
  if (workspace && !aligned16(workspace)) return PARSE_EALIGN;
  // schedule: patterns[0].schedule decides for the call (the fused single-launch kernel takes one layer only)
  const int schedule = patterns[0].schedule;
  if (schedule < PARSE_SCHED_AUTO || schedule > PARSE_SCHED_PLANNED || schedule == PARSE_SCHED_FUSED) return PARSE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  char *ws = reinterpret_cast<char *>(workspace);
  const bool planned_shapes = multi_planned_shapes(layers, patterns, n_layers) && prefill_plan_supported(P, patterns[0].n_patterns);
  const bool can_plan = planned_shapes && workspace != nullptr &&
                        workspace_bytes >= multi_planned_bytes(layers, patterns, n_layers, rows, P);
  if (schedule == PARSE_SCHED_PLANNED && !can_plan) return planned_shapes ? PARSE_EWORKSPACE : PARSE_ESHAPE;
  if (can_plan && schedule != PARSE_SCHED_TILES) {
    // planned: every layer's padded intermediate, then the plan; one plan launch, then two launches for all layers
    const int cap = prefill_plan_capacity(rows, P, patterns[0].n_patterns);
    uint16_t *Z[4];
    const int ks = prefill_planned_split(rows, args[0].n);
    for (int l = 0; l < n_layers; ++l) {
      Z[l] = reinterpret_cast<uint16_t *>(ws);
      ws += prefill_planned_z_bytes(cap, args[l].rS, ks);
    }
    int32_t *plan = reinterpret_cast<int32_t *>(ws);
    int st = build_prefill_plan(tok_offsets, pattern_id, P, rows, patterns[0].n_patterns, plan, s);
    if (st != PARSE_OK) return st;
    return forward_prefill_planned_multi_bf16(args, n_layers, plan, cap, Z, rows / P, s);
  }
  if (!tiles_ok) return PARSE_ESHAPE;
  size_t need = 0;
  for (int l = 0; l < n_layers; ++l) need += prefill_split_workspace_bytes(rows, args[l].rS);
  if (!workspace || workspace_bytes < need) return PARSE_EWORKSPACE;
  uint16_t *Z[4];
  for (int l = 0; l < n_layers; ++l) {
    Z[l] = reinterpret_cast<uint16_t *>(ws);
    ws += prefill_split_workspace_bytes(rows, args[l].rS);
  }
  return forward_prefill_split_multi_bf16(args, n_layers, Z, rows / P, s);
}

}  // extern "C"
