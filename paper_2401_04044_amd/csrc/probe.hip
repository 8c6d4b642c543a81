// Measured ceilings of the machine the library runs on, next to the datasheet peaks its
// throughput is quoted against: a pure matrix-core loop (no memory traffic at all) and a
// streaming read (16-byte loads, nothing else).  Measurement aids only: nothing on the
// split feed-forward path calls them.
#include "../../include/ffsplit.h"
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// Every wavefront issues `iters` rounds of 8 independent v_mfma_f32_32x32x16_bf16 (8
// accumulator tiles, so that the 8-pass latency of one never stalls the next).
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
probe_mfma_kernel(int iters, float* out) {
  f32x16_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  bf16x8_t a, b;
#pragma unroll
  for (int v = 0; v < 8; ++v) { a[v] = (__bf16)(float)(threadIdx.x & 3); b[v] = (__bf16)1.0f; }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  if (s == 123.456f) out[0] = s;   // never true: keeps the loop alive
}

// Grid-stride read of n16 16-byte chunks, eight loads in flight per thread, xor-reduced.
__global__ void __launch_bounds__(256) probe_read_kernel(const u32x4_t* __restrict__ p, size_t n16, uint32_t* out) {
  constexpr int U = 8;
  size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256 * U;
  u32x4_t acc = {0, 0, 0, 0};
  for (; i + (size_t)(U - 1) * 256 < n16; i += stride) {
    u32x4_t v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = p[i + (size_t)u * 256];
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u];
  }
  for (; i < n16; i += 256) acc ^= p[i];   // tail of the last sweep (only the first block's threads get here in range)
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[0] = 1;
}

}  // namespace

extern "C" {

int ffsplit_probe_mfma(int32_t workgroups, int32_t iters, void* scratch, double* flops, void* stream) {
  if (workgroups <= 0 || iters <= 0) return FFSPLIT_E_BADSHAPE;
  if (!scratch || !flops) return FFSPLIT_E_NULLPTR;
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, iters, (float*)scratch);
  if (hipGetLastError() != hipSuccess) return FFSPLIT_E_HIP;
  *flops = (double)workgroups * 4.0 * (double)iters * 8.0 * (2.0 * 32 * 32 * 16);
  return FFSPLIT_OK;
}

int ffsplit_probe_stream_read(const void* buf, size_t bytes, int32_t workgroups, void* scratch, void* stream) {
  if (workgroups <= 0 || bytes % 16 != 0) return FFSPLIT_E_BADSHAPE;
  if (!buf || !scratch) return FFSPLIT_E_NULLPTR;
  if (((uintptr_t)buf & 15u) != 0) return FFSPLIT_E_ALIGN;
  hipLaunchKernelGGL(probe_read_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (const u32x4_t*)buf,
                     bytes / 16, (uint32_t*)scratch);
  return hipGetLastError() == hipSuccess ? FFSPLIT_OK : FFSPLIT_E_HIP;
}

}  // extern "C"
