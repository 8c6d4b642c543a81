// Small-batch (at most 32 rows) bf16 products of the split feed-forward path, gfx950 only:
// the decode regime, where every product is bound by streaming its weights from HBM once.
//
//   D[M, N] = A[M, K] * Bt[N, K]^T ,  M <= 32, weights in the 32 x 16-block tiled layout.
//
// One wavefront owns one 32-row block of the weights over a range of the reduction: it
// streams that range's 1 KiB blocks (one 16-byte load per lane, contiguous across the
// wavefront), pairs each with the matching 1 KiB block of the activations (tiled, or gathered
// from a row-major matrix; they stay in cache) and feeds v_mfma_f32_32x32x16_bf16, two
// groups of eight blocks deep in registers so that about 16 KiB per wavefront is in flight.
// No LDS, no barrier.  The reduction is cut into S ranges so that a few thousand wavefronts
// exist; their fp32 partial tiles are written in accumulator order and a second kernel adds
// them in a fixed order, applies the activation and writes bf16 (tiled or row-major, one or
// two destinations) with the same column rules as the large-batch kernels' epilogue.
#include "common.h"

namespace ffsplit {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

namespace {

union SFrag {
  u32x4_t u;
  bf16x8_t v;
};

constexpr int SK_U = 8;   // blocks per register group

struct SkinnyArgs {
  const void* A;
  const void* A1;     // second left operand for odd 32-row blocks of the weights (or null)
  const void* Bt;
  int64_t lda, ldb;
  int M, N, K;
  int a_tiled;
  int n_rb;           // 32-row blocks of the weights
  int n_split;        // ranges of the reduction
  int kb_per;         // 16-element k blocks per range
  float* part;        // [n_split][n_rb][4][64] float4: accumulator order
};

template <bool A_TILED>
__global__ void __launch_bounds__(256) skinny_stream_kernel(const SkinnyArgs p) {
  const int lane = threadIdx.x & 63;
  const int task = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (task >= p.n_rb * p.n_split) return;
  const int rb = task % p.n_rb, sp = task / p.n_rb;
  const int kb_total = (p.K + 15) / 16;
  const int kb0 = sp * p.kb_per;
  const int kb1 = min(kb_total, kb0 + p.kb_per);
  const int kb_last = kb1 - 1;

  const char* wbase = (const char*)p.Bt + ((int64_t)rb * (p.ldb / 16) * 64 + lane) * 16;
  const char* abase = (const char*)((p.A1 != nullptr && (rb & 1)) ? p.A1 : p.A);
  if (A_TILED) {
    abase += (int64_t)lane * 16;
  } else {
    const int row = min(lane & 31, p.M - 1);
    abase += ((int64_t)row * p.lda + (lane >> 5) * 8) * 2;
  }
  // block kb of the weights / of the activations; past the range: the last block again (its
  // product is masked out below), so that the loads stay unconditional
  auto wload = [&](int kb) { return *(const u32x4_t*)(wbase + (int64_t)min(kb, kb_last) * 1024); };
  auto aload = [&](int kb) {
    const int k = min(kb, kb_last);
    if (A_TILED) return *(const u32x4_t*)(abase + (int64_t)k * 1024);
    // row-major: a chunk past K (K is a multiple of 8) reads the row's first chunk instead;
    // the weights are zero there
    const int col = k * 16 + (lane >> 5) * 8;
    return *(const u32x4_t*)(abase + (col < p.K ? (int64_t)k * 32 : -(int64_t)((lane >> 5) * 16)));
  };

  f32x16_t acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  u32x4_t w0[SK_U], a0[SK_U], w1[SK_U], a1[SK_U];
  if (kb0 < kb1) {
#pragma unroll
    for (int u = 0; u < SK_U; ++u) { w0[u] = wload(kb0 + u); a0[u] = aload(kb0 + u); }
    for (int kb = kb0; kb < kb1; kb += 2 * SK_U) {
#pragma unroll
      for (int u = 0; u < SK_U; ++u) { w1[u] = wload(kb + SK_U + u); a1[u] = aload(kb + SK_U + u); }
#pragma unroll
      for (int u = 0; u < SK_U; ++u) {
        SFrag w, a;
        w.u = w0[u];
        a.u = (kb + u < kb1) ? a0[u] : u32x4_t{0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w.v, a.v, acc, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < SK_U; ++u) { w0[u] = wload(kb + 2 * SK_U + u); a0[u] = aload(kb + 2 * SK_U + u); }
#pragma unroll
      for (int u = 0; u < SK_U; ++u) {
        SFrag w, a;
        w.u = w1[u];
        a.u = (kb + SK_U + u < kb1) ? a1[u] : u32x4_t{0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w.v, a.v, acc, 0, 0, 0);
      }
    }
  }
  // lane: row (token) = lane & 31; columns 8 g + 4 (lane >> 5) + 0..3 of the block in acc[4 g ..]
  float4* dst = (float4*)p.part + ((int64_t)(sp * p.n_rb + rb) * 4) * 64 + lane;
#pragma unroll
  for (int g = 0; g < 4; ++g) dst[g * 64] = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
}

__device__ __forceinline__ float sk_silu(float z) { return z / (1.0f + __expf(-z)); }

// Sum over the ranges (fixed order), activation, bf16 stores.  One thread per (block, lane,
// g): token row = lane & 31, four consecutive columns.
struct SkinnyReduceArgs {
  const float* part;
  int n_rb, n_split, M, N;
  int act, act_cols, split_col;
  void* C0;
  void* C1;
  int64_t ldc0, ldc1;
  int c0_tiled, c1_tiled, n_store;
};

__global__ void __launch_bounds__(256) skinny_reduce_kernel(const SkinnyReduceArgs p) {
  const int id = blockIdx.x * 256 + threadIdx.x;
  if (id >= p.n_rb * 256) return;
  const int rb = id >> 8, g = (id >> 6) & 3, lane = id & 63;
  const int cb = rb * 32;
  const bool act_here = cb < p.act_cols;
  const bool glu = p.act == ACT_GLU;
  int oc;
  if (glu) {
    if (act_here) {
      if (rb & 1) return;   // the pair is written from its gate block
      oc = cb / 2;
    } else {
      oc = cb - p.act_cols / 2;
    }
  } else {
    oc = cb;
  }
  auto sum_block = [&](int b) {
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    const float4* src = (const float4*)p.part + ((int64_t)b * 4 + g) * 64 + lane;
    // eight independent loads at a time, added in range order
    const int64_t step = (int64_t)p.n_rb * 256;
    for (int sp = 0; sp < p.n_split; sp += 8) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)min(sp + u, p.n_split - 1) * step];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (sp + u < p.n_split) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
    return s;
  };
  const float4 z0 = sum_block(rb);
  float v[4] = {z0.x, z0.y, z0.z, z0.w};
  if (act_here) {
    if (glu) {
      const float4 u = sum_block(rb + 1);
      const float uu[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = sk_silu(v[e]) * uu[e];
    } else if (p.act == ACT_GELU) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = gelu_f(v[e]);
    }
  }
  const int row = lane & 31;
  const int col0 = oc + 8 * g + 4 * (lane >> 5);   // first of this thread's four output columns
  char* base;
  int64_t ld;
  int col, tiled;
  if (col0 < p.split_col) { base = (char*)p.C0; ld = p.ldc0; col = col0; tiled = p.c0_tiled; }
  else { base = (char*)p.C1; ld = p.ldc1; col = col0 - p.split_col; tiled = p.c1_tiled; }
  const uint2 val = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
  if (tiled) {
    // (the destination has one 32-row block; rows past M hold repeats of row M - 1, finite)
    const int64_t chunk = ((int64_t)(col / 16) * 64) + ((col >> 3) & 1) * 32 + row;
    *(uint2*)(base + chunk * 16 + (col & 7) * 2) = val;
  } else if (row < p.M && col < p.n_store) {
    *(uint2*)(base + ((int64_t)row * ld + col) * 2) = val;
  }
}

}  // namespace

size_t skinny_part_bytes(int n_max) {
  // at most ~2048 wavefront tasks: n_rb * n_split <= 2048 + n_rb, one 4 KiB tile each
  return (size_t)(2048 + (n_max + 31) / 32) * 4096;
}

// g as for the large-batch launcher (M <= 32; destinations tiled with one row block, or
// row-major); part: scratch of skinny_part_bytes(N) bytes.
int launch_skinny_bf16(const GemmArgs& g, int act, float* part, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0) return 0;
  if (g.M > 32 || (g.N & 31) || g.partial) return -1;
  SkinnyArgs a = {};
  a.A = g.A; a.A1 = g.A1; a.Bt = g.Bt; a.lda = g.lda; a.ldb = g.ldb;
  a.M = g.M; a.N = g.N; a.K = g.K; a.a_tiled = g.a_tiled;
  a.n_rb = g.N / 32;
  const int kb_total = (g.K + 15) / 16;
  // enough ranges for about 2048 wavefronts, at least 32 blocks (32 KiB of weights) each
  int S = 2048 / a.n_rb;
  const int max_s = kb_total / 32 > 0 ? kb_total / 32 : 1;
  if (S > max_s) S = max_s;
  if (S < 1) S = 1;
  a.kb_per = (kb_total + S - 1) / S;
  a.n_split = (kb_total + a.kb_per - 1) / a.kb_per;
  a.part = part;
  const int tasks = a.n_rb * a.n_split;
  if (g.a_tiled) hipLaunchKernelGGL(skinny_stream_kernel<true>, dim3((tasks + 3) / 4), dim3(256), 0, st, a);
  else hipLaunchKernelGGL(skinny_stream_kernel<false>, dim3((tasks + 3) / 4), dim3(256), 0, st, a);
  if (hipGetLastError() != hipSuccess) return -1;
  SkinnyReduceArgs r = {};
  r.part = part; r.n_rb = a.n_rb; r.n_split = a.n_split; r.M = g.M; r.N = g.N;
  r.act = act; r.act_cols = g.act_cols; r.split_col = g.split_col;
  r.C0 = g.C0; r.C1 = g.C1; r.ldc0 = g.ldc0; r.ldc1 = g.ldc1;
  r.c0_tiled = g.c0_tiled; r.c1_tiled = g.c1_tiled; r.n_store = g.n_store;
  hipLaunchKernelGGL(skinny_reduce_kernel, dim3(a.n_rb), dim3(256), 0, st, r);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace ffsplit
