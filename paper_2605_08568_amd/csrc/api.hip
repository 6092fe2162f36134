// Status strings, host-side validators and the checks shared by every entry point.
#include <stdio.h>
#include <string.h>

#include "common.hpp"

namespace parse {

static thread_local char g_hip_error[256] = "no HIP error recorded";

void set_hip_error(hipError_t e, const char *where) {
  snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", where, hipGetErrorString(e));
}

int check_layer(const parse_layer *L) {
  if (!L || !L->Vt || !L->Ut) return PARSE_EINVAL;
  if (L->dtype != PARSE_F32 && L->dtype != PARSE_BF16) return PARSE_EINVAL;
  if (L->layout != PARSE_ROWMAJOR && L->layout != PARSE_MFMA16) return PARSE_EINVAL;
  if (L->n <= 0 || L->m <= 0 || L->R <= 0 || L->G <= 0) return PARSE_EINVAL;
  if (L->R % L->G != 0) return PARSE_ESHAPE;
  if (!aligned16(L->Vt) || !aligned16(L->Ut)) return PARSE_EALIGN;
  const int per16 = 16 / elem_size(L->dtype);
  if (L->n % per16 != 0 || L->m % per16 != 0) return PARSE_EALIGN;
  if (L->layout == PARSE_MFMA16) {
    if (L->dtype != PARSE_BF16) return PARSE_ELAYOUT;
    const int gs = L->R / L->G;
    if (L->n % 16 != 0 || L->m % 32 != 0 || gs % 32 != 0) return PARSE_ESHAPE;
  }
  return PARSE_OK;
}

}  // namespace parse

extern "C" {

const char *parse_status_string(int status) {
  switch (status) {
    case PARSE_OK: return "ok";
    case PARSE_EINVAL: return "invalid argument (NULL pointer, bad enum or non-positive size)";
    case PARSE_ESHAPE: return "shape mismatch or size outside the kernel's limits";
    case PARSE_EALIGN: return "pointer or leading dimension not 16-byte aligned";
    case PARSE_ECAPACITY: return "pattern cache is full";
    case PARSE_EWORKSPACE: return "workspace missing or too small";
    case PARSE_EHIP: return "HIP runtime error (see parse_last_hip_error)";
    case PARSE_ELAYOUT: return "factor layout not supported by this call";
    default: return "unknown status";
  }
}

const char *parse_last_hip_error(void) { return parse::g_hip_error; }

int parse_version(void) { return 100; }

int parse_check_offsets(const int32_t *off, int32_t P, int32_t rows) {
  if (!off || P <= 0 || rows <= 0) return PARSE_EINVAL;
  if (off[0] != 0 || off[P] != rows) return PARSE_ESHAPE;
  for (int32_t p = 0; p < P; ++p)
    if (off[p + 1] <= off[p]) return PARSE_ESHAPE;
  return PARSE_OK;
}

int parse_check_subset(const int32_t *subset, int32_t k, int32_t G) {
  if (!subset || k <= 0 || G <= 0) return PARSE_EINVAL;
  if (k > G) return PARSE_ESHAPE;
  for (int32_t i = 0; i < k; ++i) {
    if (subset[i] < 0 || subset[i] >= G) return PARSE_ESHAPE;
    if (i > 0 && subset[i] <= subset[i - 1]) return PARSE_ESHAPE;
  }
  return PARSE_OK;
}

}  // extern "C"
