// parse_lowrank_decode_static: the decode step for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  It is parse_lowrank_forward(PARSE_DECODE)
// with the workspace replaced by a fixed array in the library's own device image: no hipMalloc, no hipFree, no
// allocating library routine on any call, including the first.
#include <mutex>

#include "common.hpp"

namespace parse {
size_t decode_workspace_bytes(const parse_layer *L);
int forward_decode_bf16(const parse_layer *L, const parse_patterns *pt, const uint16_t *x, int B,
                        const int32_t *pattern_id, uint16_t *y, void *workspace, hipStream_t s);
}  // namespace parse

using namespace parse;

// Every GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
// In host code the array's NAME is only a stand-in for the symbol: the address the kernels can use is the one
// hipGetSymbolAddress returns for the current device, kept in scratch_of[] below.
static __device__ __align__(256) unsigned char scratch[PARSE_DECODE_STATIC_SCRATCH_BYTES];

static std::mutex scratch_mutex;
static void *scratch_of[64] = {nullptr};   // per device: the device address of that device's copy

// Device address of the current device's scratch array (looked up once per device, with that device current).
static int scratch_address(void **out) {
  int dev = 0;
  PARSE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return PARSE_EINVAL;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_of[dev]) {
    void *ptr = nullptr;
    PARSE_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return PARSE_EHIP;
    scratch_of[dev] = ptr;
  }
  *out = scratch_of[dev];
  return PARSE_OK;
}

extern "C" {

size_t parse_lowrank_decode_static_capacity(void) { return (size_t)PARSE_DECODE_STATIC_SCRATCH_BYTES; }

int parse_lowrank_decode_static(const parse_layer *L, const parse_patterns *pt, const void *X, int32_t rows,
                                const int32_t *pattern_id, void *Y, parse_stream stream) {
  int st = check_layer(L);
  if (st != PARSE_OK) return st;
  if (!pt || !X || !Y || !pattern_id || !pt->subsets) return PARSE_EINVAL;
  if (rows <= 0 || pt->n_patterns <= 0 || pt->k <= 0) return PARSE_EINVAL;
  if (L->dtype != PARSE_BF16 || L->layout != PARSE_MFMA16) return PARSE_ELAYOUT;
  if (pt->k > L->G || rows > 32 || L->G > 64 || pt->subset_stride < pt->k) return PARSE_ESHAPE;
  if (!aligned16(X) || !aligned16(Y)) return PARSE_EALIGN;
  // what the decode kernels need beyond inputs and outputs must fit the fixed array
  if (decode_workspace_bytes(L) > (size_t)PARSE_DECODE_STATIC_SCRATCH_BYTES) return PARSE_EWORKSPACE;
  void *ws = nullptr;
  st = scratch_address(&ws);
  if (st != PARSE_OK) return st;
  // What has to start at zero -- the arrival counters of the split reduction -- is part of the decode plan, which the
  // call builds into the array first (a small kernel, no memset); every partial sum and every list entry the kernels
  // read in a call was written earlier in that same call (the previous call's contents are overwritten or never looked at).
  return forward_decode_bf16(L, pt, (const uint16_t *)X, rows, pattern_id, (uint16_t *)Y, ws, (hipStream_t)stream);
}

}  // extern "C"
