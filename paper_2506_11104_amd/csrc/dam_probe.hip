// Two measurement kernels for the roofline lines of the benchmark: what this chip sustains when a kernel does
// nothing but bf16 matrix instructions, and nothing but streaming reads. They are the denominators "measured on
// the box" that stand next to the published peaks; nothing of the method is computed here.
#include <hip/hip_runtime.h>

#include "dam_internal.h"

namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Every wave holds four A and four B fragments (operand data from memory, so that the multipliers see real bit
// patterns) and runs 16 v_mfma_f32_32x32x16_bf16 per loop pass into four independent accumulators, the
// instruction mix of an attention kernel's inner loop without anything else. Two workgroups of four waves per CU
// put two waves on every SIMD.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_probe_mfma(
    const uint4 *__restrict__ operands, float *__restrict__ sink, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    a[j] = __builtin_bit_cast(bf16x8, operands[(j * 64 + lane) & 511]);
    b[j] = __builtin_bit_cast(bf16x8, operands[((j + 4) * 64 + lane) & 511]);
  }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + r) & 3], acc[j], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[j][e];
  if (s == 12345.678f) sink[0] = s;  // keeps the products alive; practically never true
}

// 16-byte non-temporal loads, eight in flight per lane, grid-stride over the buffer.
__global__ __launch_bounds__(256) void k_probe_read(const uint4 *__restrict__ src, size_t n, unsigned *__restrict__ sink) {
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
  constexpr int U = 8;
  size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256 * U;
  unsigned acc = 0;
  for (; i + 256 * (U - 1) < n; i += stride) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src) + i + 256 * u);
#pragma unroll
    for (int u = 0; u < U; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x12345678u) sink[0] = acc;
}
}  // namespace

extern "C" int dam_probe_mfma(const void *operands, float *sink, int32_t workgroups, int32_t iters, void *stream) {
  if (!operands || !sink || workgroups < 1 || iters < 1) return DAM_ERR_INVALID_ARG;
  k_probe_mfma<<<workgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const uint4 *>(operands), sink, iters);
  return dam::launch_status();
}

extern "C" int dam_probe_stream_read(const void *src, size_t bytes, uint32_t *sink, int32_t workgroups, void *stream) {
  if (!src || !sink || workgroups < 1 || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15)) return DAM_ERR_INVALID_ARG;
  k_probe_read<<<workgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const uint4 *>(src), bytes / 16, sink);
  return dam::launch_status();
}
