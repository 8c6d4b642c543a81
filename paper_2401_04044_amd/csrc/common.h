// Internal declarations shared by the HIP translation units of libffsplit.
// Nothing here is part of the C ABI (that is include/ffsplit.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace ffs {

typedef uint16_t bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// round-to-nearest-even fp32 -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// exact GeLU z * Phi(z) (Sec. 2 cites it as the FFN activation)
__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
// SiLU z * sigmoid(z), the SwiGLU gate non-linearity
__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

enum { ACT_NONE = 0, ACT_GELU = 1, ACT_GLU = 2 };

// Exclusive prefix count of `flag` over the 1024 threads of a block, in thread
// order, plus the block total.  wsum: 16 ints of LDS.  Every thread must call it.
__device__ __forceinline__ int block_prefix_1024(bool flag, int* wsum, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long m = __ballot(flag);
  const int within = __popcll(m & ((1ull << lane) - 1ull));
  __syncthreads();
  if (lane == 0) wsum[wave] = __popcll(m);
  __syncthreads();
  int before = 0, tot = 0;
  for (int w = 0; w < 16; ++w) {
    const int c = wsum[w];
    if (w < wave) before += c;
    tot += c;
  }
  *total = tot;
  return before + within;
}

// One GEMM launch:  D[M, N] = A[M, K] * Bt[N, K]^T  followed by an epilogue.
// A and Bt are K-contiguous.  With dual_a, 32-column blocks alternate between
// A (even blocks) and A1 (odd blocks) as the left operand.
struct GemmArgs {
  const void* A;
  const void* A1;
  const void* Bt;
  int64_t lda, ldb;
  int M, N, K;
  // epilogue
  // Columns [0, act_cols) get the activation; with ACT_GLU they are (gate, up)
  // pairs of 32-column blocks and produce act_cols/2 output columns.
  // Output column c (after pairing) goes to C0[:, c] if c < split_col else to
  // C1[:, c - split_col].
  int act_cols;
  int split_col;
  void* C0;
  void* C1;
  int64_t ldc0, ldc1;
  int out_f32;     // bf16 kernels only: store fp32 instead of bf16
  // score mode: per-row-tile partial column sums of h^2 and |h|
  float* part_s2;  // [tiles_m, n_out]
  float* part_s1;
  int n_out;
};

int launch_gemm(const GemmArgs& a, int dtype_bf16, int act, bool score, hipStream_t st);
int gemm_tile_m(int dtype_bf16);  // rows per score partial

}  // namespace ffs
