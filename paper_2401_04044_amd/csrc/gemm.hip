// fp32 GEMM of the split feed-forward path (the bf16 MFMA kernel is gemm_bf16.hip).
//
//   D[M, N] = A[M, K] * Bt[N, K]^T        (both operands row-major, K-contiguous)
//
// followed by one of the fused epilogues the path needs:
//   - store (optionally exact GeLU, or SwiGLU on (gate, up) pairs of 32-column
//     blocks), with the output columns routed to two destinations;
//   - score: per-row-tile column sums of h^2 and |h| (the neuron-norm reduction
//     of Sec. 4.1, Eq. 3), h never leaving registers.
// Plain FMA tiles: the fp32 workload is tiny and latency-bound, and its 1e-5
// error bar wants true fp32 products and the erf form of GeLU.
#include "common.h"

namespace ffsplit {

// ------------------------------------------------------------------ fp32 FMA kernel
// 64x64 tile, 16-deep K slabs, 256 threads; thread (ty, tx) owns rows ty + 16 i
// and columns tx + 16 j (i, j = 0..3), so that column j and j + 2 are a
// (gate, up) pair of 32-column blocks.

template <int ACT, bool DUAL, bool SCORE>
__global__ void __launch_bounds__(256) gemm_f32_kernel(const GemmArgs p) {
  constexpr int BM = 64, BN = 64, BK = 16, LD = 65;
  constexpr int NA = DUAL ? 2 : 1;
  __shared__ float sA[NA][BK][LD];
  __shared__ float sB[BK][LD];
  __shared__ float red[2][16][BN];

  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;

  const int lrow = tid >> 2, lk = (tid & 3) * 4;
  int ga = m0 + lrow;
  ga = ga < p.M ? ga : p.M - 1;
  int gb = n0 + lrow;
  gb = gb < p.N ? gb : p.N - 1;
  const float* a_src[NA] = {(const float*)p.A + (int64_t)ga * p.lda + lk};
  if (DUAL) a_src[NA - 1] = (const float*)p.A1 + (int64_t)ga * p.lda + lk;
  const float* b_src = (const float*)p.Bt + (int64_t)gb * p.ldb + lk;

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  // gridDim.y > 1 (only with p.partial): this workgroup's range of the reduction, whole slabs
  const int slabs = (p.K + BK - 1) / BK;
  const int per = (slabs + (int)gridDim.y - 1) / (int)gridDim.y;
  const int k_begin = (int)blockIdx.y * per * BK;
  const int k_end = min(p.K, k_begin + per * BK);
  // the next slab's global loads are in flight while this one is multiplied
  float4 va[NA], vb;
  auto fetch = [&](int k0) {
    const bool ok = k0 < k_end && (k0 + lk) < p.K;
#pragma unroll
    for (int s = 0; s < NA; ++s) va[s] = ok ? *(const float4*)(a_src[s] + k0) : make_float4(0, 0, 0, 0);
    vb = ok ? *(const float4*)(b_src + k0) : make_float4(0, 0, 0, 0);
  };
  fetch(k_begin);
  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
    __syncthreads();
#pragma unroll
    for (int s = 0; s < NA; ++s) {
      sA[s][lk + 0][lrow] = va[s].x; sA[s][lk + 1][lrow] = va[s].y;
      sA[s][lk + 2][lrow] = va[s].z; sA[s][lk + 3][lrow] = va[s].w;
    }
    sB[lk + 0][lrow] = vb.x; sB[lk + 1][lrow] = vb.y; sB[lk + 2][lrow] = vb.z; sB[lk + 3][lrow] = vb.w;
    __syncthreads();
    fetch(k0 + BK);
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[NA][4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int s = 0; s < NA; ++s) a[s][i] = sA[s][k][ty + 16 * i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = sB[k][tx + 16 * j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[DUAL ? (j >> 1) : 0][i], b[j], acc[i][j]);
    }
  }

  // output column (after GLU pairing) of local column block
  const bool glu_here = (ACT == ACT_GLU) && (n0 < p.act_cols);
  if (!SCORE) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (glu_here && j >= 2) continue;
      const int cb = n0 + tx + 16 * j;
      if (cb >= p.N) continue;
      int oc;
      if (ACT == ACT_GLU) oc = glu_here ? (n0 / 2 + tx + 16 * j) : cb - p.act_cols / 2;
      else oc = cb;
      float* base;
      int64_t ld;
      if (oc < p.split_col) { base = (float*)p.C0 + oc; ld = p.ldc0; }
      else { base = (float*)p.C1 + (oc - p.split_col); ld = p.ldc1; }
      if (p.partial) base += (int64_t)blockIdx.y * p.M * p.ldc0;   // fp32 partials [split][M][ldc0]
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = m0 + ty + 16 * i;
        if (row >= p.M) continue;
        float v;
        // (a neuron's bias before the activation; the output bias of an un-activated product)
        const float bz = (ACT != ACT_GLU && p.bias != nullptr && cb < p.bias_cols) ? p.bias[cb] : 0.f;
        if (ACT == ACT_GLU) v = glu_here ? silu_f(acc[i][j]) * acc[i][(j + 2) & 3] : acc[i][j];
        else if (ACT == ACT_GELU) v = cb < p.act_cols ? gelu_f(acc[i][j] + bz) : acc[i][j] + bz;
        else v = acc[i][j] + bz;
        if (p.resid != nullptr && !p.partial && oc < p.split_col) v += p.resid[(int64_t)row * p.ldr + oc];
        base[(int64_t)row * ld] = v;
      }
    }
  } else {
    constexpr int NJ = (ACT == ACT_GLU) ? 2 : 4;
    constexpr int BNO = (ACT == ACT_GLU) ? 32 : 64;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      float s2 = 0.f, s1 = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = m0 + ty + 16 * i;
        float h = (ACT == ACT_GLU) ? silu_f(acc[i][j]) * acc[i][j + 2] : gelu_f(acc[i][j]);
        h = row < p.M ? h : 0.f;
        s2 += h * h;
        s1 += fabsf(h);
      }
      red[0][ty][tx + 16 * j] = s2;
      red[1][ty][tx + 16 * j] = s1;
    }
    __syncthreads();
    if (tid < BNO) {
      const int col = n0 / ((ACT == ACT_GLU) ? 2 : 1) + tid;
      if (col < p.n_out) {
        float a2 = 0.f, a1 = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) { a2 += red[0][w][tid]; a1 += red[1][w][tid]; }
        p.part_s2[(int64_t)tm * p.n_out + col] = a2;
        p.part_s1[(int64_t)tm * p.n_out + col] = a1;
      }
    }
  }
}

// Sum of fp32 partials [n_split][M][ldp] of a whole product (GEMM column order, written with
// a.partial and no activation) followed by the store epilogue of gemm_f32_kernel: bias,
// activation (exact GeLU, or SwiGLU on (gate, up) pairs of 32-column blocks), routing to two
// fp32 destinations, residual.  One thread per (row, output column), columns fastest.
struct SplitEpiF32Args {
  const float* part;
  int n_split, M, ldp, n_out;
  int act, act_cols, split_col;
  float* C0;
  float* C1;
  int64_t ldc0, ldc1;
  const float* bias;
  int bias_cols;
  const float* resid;
  int64_t ldr;
};

__global__ void __launch_bounds__(256) splitk_epilogue_f32_kernel(const SplitEpiF32Args p) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= (int64_t)p.M * p.n_out) return;
  const int row = (int)(id / p.n_out), oc = (int)(id % p.n_out);
  const bool glu = p.act == ACT_GLU;
  const bool pair = glu && oc < p.act_cols / 2;
  int c = oc;   // GEMM column of the (gate) value
  if (glu) c = pair ? (oc / 32) * 64 + (oc & 31) : oc + p.act_cols / 2;
  float v = 0.f, u = 0.f;
  for (int s = 0; s < p.n_split; ++s) {
    const float* src = p.part + ((int64_t)s * p.M + row) * p.ldp + c;
    v += src[0];
    if (pair) u += src[32];
  }
  if (!glu && p.bias != nullptr && c < p.bias_cols) v += p.bias[c];
  if (pair) v = silu_f(v) * u;
  else if (p.act == ACT_GELU && c < p.act_cols) v = gelu_f(v);
  if (oc < p.split_col) {
    if (p.resid != nullptr) v += p.resid[(int64_t)row * p.ldr + oc];
    p.C0[(int64_t)row * p.ldc0 + oc] = v;
  } else {
    p.C1[(int64_t)row * p.ldc1 + (oc - p.split_col)] = v;
  }
}

int launch_splitk_epilogue_f32(const float* part, int n_split, int ldp, const GemmArgs& g, int act, hipStream_t st) {
  SplitEpiF32Args a = {};
  a.part = part; a.n_split = n_split; a.M = g.M; a.ldp = ldp;
  a.n_out = act == ACT_GLU ? g.N - g.act_cols / 2 : g.N;
  a.act = act; a.act_cols = g.act_cols; a.split_col = g.split_col;
  a.C0 = (float*)g.C0; a.C1 = (float*)g.C1; a.ldc0 = g.ldc0; a.ldc1 = g.ldc1;
  a.bias = g.bias; a.bias_cols = g.bias_cols; a.resid = g.resid; a.ldr = g.ldr;
  if (act == ACT_GLU && (g.act_cols & 63)) return -1;
  const int64_t n = (int64_t)a.M * a.n_out;
  if (n <= 0) return 0;
  hipLaunchKernelGGL(splitk_epilogue_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ------------------------------------------------------------------ host launchers

template <int ACT, bool DUAL, bool SCORE>
static int launch_f32(const GemmArgs& a, int n_split, hipStream_t st) {
  const int tiles = ((a.M + 63) / 64) * ((a.N + 63) / 64);
  hipLaunchKernelGGL((gemm_f32_kernel<ACT, DUAL, SCORE>), dim3(tiles, n_split), dim3(256), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_gemm_f32(const GemmArgs& a, int act, bool score, hipStream_t st, int n_split) {
  if (a.M <= 0 || a.N <= 0) return 0;
  const bool dual = a.A1 != nullptr;
  if (n_split > 1 && !(a.partial && act == ACT_NONE && !score)) return -1;
  if (score) {
    if (act == ACT_GELU) return launch_f32<ACT_GELU, false, true>(a, 1, st);
    if (act == ACT_GLU) return launch_f32<ACT_GLU, false, true>(a, 1, st);
    return -1;
  }
  if (act == ACT_NONE) return launch_f32<ACT_NONE, false, false>(a, n_split, st);
  if (act == ACT_GELU) return launch_f32<ACT_GELU, false, false>(a, 1, st);
  if (act == ACT_GLU && !dual) return launch_f32<ACT_GLU, false, false>(a, 1, st);
  if (act == ACT_GLU && dual) return launch_f32<ACT_GLU, true, false>(a, 1, st);
  return -1;
}

}  // namespace ffsplit
