// Achievable-peak probes: what this machine sustains on the two resources the hot path is priced against, measured
// with kernels of the same kind as the product's (same matrix instruction, same 16-byte-per-lane streams), so that a
// roofline fraction can be read against the nominal peak AND against what a kernel with no other work reaches.
//   parse_probe_mfma_bf16   register-resident loop of 32x32x16 bf16 matrix instructions on the caller's data
//                           (8 independent accumulators per wavefront, 4 wavefronts per workgroup, no memory traffic
//                           inside the loop).  The rate depends on the DATA (switching activity): random bf16 values
//                           run slower than constants on a power-limited part.
//   parse_probe_read        read-only stream: every workgroup reads its contiguous share with 16-byte loads that write
//                           LDS directly (1 KiB per wavefront instruction, many in flight), nothing is written.
//   parse_probe_copy        plain copy, 16 bytes per lane (the known-size kernel the traffic counters are scaled by).
// The caller times them (HIP events on its stream); they only enqueue.
#include "common.hpp"

namespace parse {

__global__ __launch_bounds__(256) void probe_mfma(const u32x4 *__restrict__ in, float *__restrict__ out, int iters) {
  u32x4 a[4], b[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = in[threadIdx.x + 256 * i];
#pragma unroll
  for (int i = 0; i < 2; ++i) b[i] = in[threadIdx.x + 256 * (4 + i)];
  f32x16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[j % 4]), __builtin_bit_cast(bf16x8, b[j % 2]),
                                                       acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[j][e];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

constexpr int PR_WAVES = 8, PR_DEPTH = 8;   // 8 wavefronts x 8 KiB = 64 KiB of LDS landing space per workgroup

__global__ __launch_bounds__(PR_WAVES * 64) void probe_read(const char *__restrict__ src, size_t bytes_per_wg, uint32_t *sink) {
  __shared__ __attribute__((aligned(1024))) char lds[PR_WAVES * PR_DEPTH * 1024];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const size_t per_wave = bytes_per_wg / PR_WAVES;
  const char *p = src + (size_t)blockIdx.x * bytes_per_wg + (size_t)wave * per_wave + lane * 16;
  for (size_t o = 0; o + PR_DEPTH * 1024 <= per_wave; o += PR_DEPTH * 1024) {
#pragma unroll
    for (int i = 0; i < PR_DEPTH; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p + o + i * 1024),
                                       (__attribute__((address_space(3))) void *)(lds + (wave * PR_DEPTH + i) * 1024), 16, 0, 0);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PR_DEPTH) : "memory");   // at most two batches in flight
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  const uint32_t v = *reinterpret_cast<const uint32_t *>(lds + threadIdx.x * 16);
  if (v == 0x9E3779B9u && sink) sink[0] = v;   // keeps the reads alive; practically never true
}

__global__ __launch_bounds__(256) void probe_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace parse

using namespace parse;

extern "C" {

int parse_probe_mfma_bf16(const void *data, int32_t workgroups, int32_t iters, float *out, parse_stream stream) {
  if (!data || !out) return PARSE_EINVAL;
  if (workgroups <= 0 || iters <= 0) return PARSE_EINVAL;
  if (!aligned16(data)) return PARSE_EALIGN;
  hipLaunchKernelGGL(probe_mfma, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)data, out, iters);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

int parse_probe_read(const void *src, size_t bytes, int32_t workgroups, void *sink, parse_stream stream) {
  if (!src) return PARSE_EINVAL;
  if (workgroups <= 0 || bytes == 0) return PARSE_EINVAL;
  if (!aligned16(src)) return PARSE_EALIGN;
  const size_t quantum = (size_t)PR_WAVES * PR_DEPTH * 1024;
  if (bytes % ((size_t)workgroups * quantum) != 0) return PARSE_ESHAPE;   // whole 64 KiB batches per workgroup
  hipLaunchKernelGGL(probe_read, dim3(workgroups), dim3(PR_WAVES * 64), 0, (hipStream_t)stream, (const char *)src,
                     bytes / workgroups, (uint32_t *)sink);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

int parse_probe_copy(const void *src, void *dst, size_t bytes, parse_stream stream) {
  if (!src || !dst) return PARSE_EINVAL;
  if (bytes == 0 || bytes % 16 != 0) return PARSE_ESHAPE;
  if (!aligned16(src) || !aligned16(dst)) return PARSE_EALIGN;
  hipLaunchKernelGGL(probe_copy, dim3(2048), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)src, (u32x4 *)dst, bytes / 16);
  PARSE_LAUNCH_CHECK();
  return PARSE_OK;
}

}  // extern "C"
