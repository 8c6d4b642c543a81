// Internal declarations shared by the HIP translation units of libffsplit.
// Nothing here is part of the C ABI (that is include/ffsplit.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace ffsplit {

typedef uint16_t bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// round-to-nearest-even fp32 -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// two fp32 -> packed bf16 pair, round-to-nearest-even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const bf16x2_t r = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
  uint32_t u;
  __builtin_memcpy(&u, &r, 4);
  return u;
}

// exact GeLU z * Phi(z) (Sec. 2 cites it as the FFN activation)
__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
// SiLU z * sigmoid(z), the SwiGLU gate non-linearity
__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// GeLU for the bf16 path with one transcendental: for a = |z|, Phi(-a) = 2^q(a) with q a cubic
// fitted to log2 Phi(-a) (leading coefficient negative, so large a underflows to 0), and
// z Phi(z) = max(z, 0) - a Phi(-a).  Max abs error 5.7e-5 on the real line, below the bf16
// rounding of the result (2^-9 relative) wherever |result| > 0.03.
__device__ __forceinline__ float gelu_fast(float z) {
  const float a = fabsf(z);
  float q = fmaf(a, -0.024829373f, -0.49904245f);
  q = fmaf(a, q, -1.1289980f);
  q = fmaf(a, q, -1.0036056f);
  return fmaxf(z, 0.0f) - a * __builtin_amdgcn_exp2f(q);
}
__device__ __forceinline__ float silu_fast(float z) {
  const float e = __builtin_amdgcn_exp2f(-1.44269504f * z);
  return z * __builtin_amdgcn_rcpf(1.0f + e);
}

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
// fp32 kernels: A and Bt row-major, K-contiguous.  bf16 kernels: Bt in the tiled
// layout (see gemm_bf16.hip), A row-major or tiled, outputs row-major or tiled.
// With A1 set, 32-column blocks alternate between A (even blocks) and A1 (odd
// blocks) as the left operand.
struct GemmArgs {
  const void* A;
  const void* A1;
  const void* Bt;
  int64_t lda, ldb;   // row-major: elements per row; tiled: padded K of the buffer
  int M, N, K;
  int a_tiled;
  int group_m;     // bf16 kernels: row tiles per rasterisation group (>= 1)
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
  int c0_tiled, c1_tiled;
  int m_pad;       // rows of a tiled destination (multiple of 32)
  int n_store;     // valid columns of a row-major destination
  int partial;     // bf16 kernels: write fp32 split-K partials [split][M][ldc0] to C0 instead
  // Optional additions of the store epilogue (never with partial):
  //   bias [bias_cols] fp32, added to GEMM columns [0, bias_cols) before the activation (a
  //   neuron's bias; not with ACT_GLU), or to every output column of an un-activated product;
  //   resid [M, ldr] fp32, added to the value routed to C0 (row-major destinations only);
  //   out_f32: C0 holds fp32 [M, ldc0] instead of the storage type.
  const float* bias;
  int bias_cols;
  const float* resid;
  int64_t ldr;
  int out_f32;
  // score mode: per-row-tile partial column sums of h^2 and |h|
  float* part_s2;  // [tiles_m, n_out]
  float* part_s1;
  int n_out;
};

// What a forward call adds around the two halves of Eq. 2 (all optional): the neurons' biases in
// packed order [heavy kp | remainder mp] (fp32), the output bias [d_model] (fp32), the residual
// stream [T, d_model] (fp32) and an fp32 destination for Y.
struct Epilogue {
  const float* b1;
  const float* b2;
  const float* resid;
  int out_f32;
};

// n_split > 1: only with a.partial and no activation: fp32 partials [split][M][ldc0] into C0
int launch_gemm_f32(const GemmArgs& a, int act, bool score, hipStream_t st, int n_split = 1);
// sum of fp32 partials [n_split][a.M][ldp] of a whole product + the fp32 store epilogue described by a
int launch_splitk_epilogue_f32(const float* part, int n_split, int ldp, const GemmArgs& a, int act, hipStream_t st);
// tile configurations of the bf16 kernel
enum {
  GEMM_256x128 = 0,        // 4 wavefronts, 3 stages: the default for large products
  GEMM_128x128 = 1,        // 4 wavefronts, 3 stages: small or narrow products
  GEMM_128x128_KSPLIT = 2, // 8 wavefronts, 64-deep slabs, reduction split inside the workgroup (few tiles)
  GEMM_256x256 = 3,        // 8 wavefronts, 3 stages
  GEMM_256x320 = 4,        // 4 wavefronts, wave tile 128 x 160 (one wavefront per SIMD): N a multiple of 320
  GEMM_128x320 = 5,        // 4 wavefronts, wave tile 64 x 160
  GEMM_256x256_W64 = 6     // 8 wavefronts as 4 x 2, wave tile 64 x 128: fewer reads of two left operands
};
// n_split > 1 only with a.partial
int launch_gemm_bf16(const GemmArgs& a, int act, bool score, int shape, int n_split, hipStream_t st);
// sum of the partials in a fixed order -> C (bf16, tiled or row-major; f32_out: fp32 row-major)
int launch_splitk_reduce(const float* part, int n_split, int M, int N, int m_pad, void* C, int64_t ldc, int tiled,
                         hipStream_t st, int f32_out = 0);
// sum of the fp32 partials [n_split][a.M][ldp] of a whole product (written with a.partial, no
// activation, GEMM column order) + the store epilogue described by a (activation act)
int launch_splitk_epilogue(const float* part, int n_split, int ldp, const GemmArgs& a, int act, hipStream_t st);
int bf16_score_tile_m();
// The two middle products of the low-rank remainder in one launch (ffn2_fused.hip):
// part[n_split][M][512] = per neuron range, gelu(T1 * Q1t^T) * P2t^T, all operands tiled bf16 with
// the padded reduction lengths given (ldt, ldq = 512 = rp; ldp2 = mp, a multiple of 64).
// n_split must be ffn2_fused_splits(M, mp).  Returns 0, -1 on an error, 1 where the device does
// not grant the LDS the kernel needs (nothing launched).
constexpr int FFN2_FUSED_RANK = 512;
int ffn2_fused_splits(int M, int mp);
int launch_ffn2_fused(const void* T1, int64_t ldt, const void* Q1t, int64_t ldq, const void* P2t, int64_t ldp2, int M,
                      int mp, int rp, float* part, int n_split, hipStream_t st);
// small-batch path (M <= SKINNY_MAX_M, N a multiple of 32): weight-streaming kernels, one or two
// blocks of 32 tokens per pass over the weights (four blocks were measured no better than the
// tiled GEMM at 128 rows); part: scratch of skinny_part_bytes(N, M) bytes
constexpr int SKINNY_MAX_M = 64;
size_t skinny_part_bytes(int n_max, int M);
int launch_skinny_bf16(const GemmArgs& a, int act, float* part, hipStream_t st);
// the reduce half alone: sum of n_split ranges of partial tiles, activation, stores
// (f16_out: the destinations hold fp16, saturating, instead of bf16)
int launch_skinny_reduce(const GemmArgs& a, int act, const float* part, int n_split, int f16_out, hipStream_t st);
// weights of one product in the quantised tiled format (qformat.h)
struct SkinnyQ {
  const void* codes;
  const void* scales;
  int bits;   // 8 or 3
  int down;   // 0: one scale per (row, 128 reduction elements), [row block][G][32];
              // 1: one per (128 rows, reduction element), [rows / 128][Kp]
  int G, Kp;
};
// One product whose weights are part 8-bit (g8, q8), part 3-bit (g3, q3), in one launch; a part
// with N = 0 or K = 0 is absent.  M <= 32, K a multiple of 64.
//   up   (q.down = 0): A = the caller's row-major bf16 X, K a multiple of 128; the two parts
//        are two row ranges of one output (8-bit rows first): partial tiles
//        [range][g8.N / 32 + g3.N / 32 row blocks], n_split[0] ranges for the first rows,
//        n_split[1] for the others (launch_skinny_reduce2).
//   down (q.down = 1): A tiled fp16 with one row block; the two parts are two segments of the
//        reduction over the same N rows: partial tiles of ranges [0, n_split[0]) and
//        [n_split[0], n_split[0] + n_split[1]).
// part: skinny_q_part_bytes(N) bytes.
size_t skinny_q_part_bytes(int n_max);
int launch_skinny_q_pair(const GemmArgs& g8, const SkinnyQ& q8, const GemmArgs& g3, const SkinnyQ& q3, float* part,
                         int n_split[2], hipStream_t st);
// reduce with n_split ranges for row blocks below rb_split and n_split_b from there on
int launch_skinny_reduce2(const GemmArgs& a, int act, const float* part, int n_split, int rb_split, int n_split_b,
                          int f16_out, hipStream_t st);

}  // namespace ffsplit
