// GEMM kernels of the split feed-forward path, for gfx950 only.
//
//   D[M, N] = A[M, K] * Bt[N, K]^T        (both operands K-contiguous)
//
// followed by one of the fused epilogues the path needs:
//   - store (optionally GeLU, or SwiGLU on (gate, up) pairs of 32-column blocks),
//     with the output columns routed to two destinations;
//   - score: per-row-tile column sums of h^2 and |h| (the neuron-norm reduction
//     of Sec. 4.1, Eq. 3), h never leaving registers.
//
// bf16: v_mfma_f32_32x32x16_bf16, LDS-staged 64-deep K slabs, XOR-swizzled 16-byte
//       chunks, register prefetch of the next slab, fp32 accumulation.
// fp32: plain FMA tiles (the fp32 workload is tiny and latency-bound).
#include "common.h"

namespace ffs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

union Frag {
  uint4 u;
  bf16x8_t v;
};

// Workgroup i of the grid runs on XCD i % 8; give each XCD a contiguous run of
// logical tiles so that neighbours in tile order share an L2.
__device__ __forceinline__ int xcd_remap(int i, int total) {
  const int q = total >> 3, rem = total & 7, x = i & 7;
  return x * q + (x < rem ? x : rem) + (i >> 3);
}

template <int ACT>
__device__ __forceinline__ float apply_act(float z, float g) {
  if (ACT == ACT_GELU) return gelu_f(z);
  if (ACT == ACT_GLU) return silu_f(g) * z;
  return z;
}

// ------------------------------------------------------------------ bf16 MFMA kernel

template <int BM, int BN, int WGM, int WGN, int ACT, bool DUAL, bool SCORE>
__global__ void __launch_bounds__(WGM* WGN * 64) gemm_bf16_kernel(const GemmArgs p) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int NA = DUAL ? 2 : 1;
  constexpr int CA = BM * 8 / NT, CB = BN * 8 / NT;
  constexpr int STAGE = (NA * BM + BN) * 8;  // uint4 per stage
  constexpr bool SWAP = !SCORE;              // SWAP: lanes hold 4 consecutive output columns
  static_assert(ACT != ACT_GLU || (TN % 2 == 0), "GLU needs paired column blocks per wave");
  static_assert(!DUAL || ACT == ACT_GLU, "dual left operand only for GLU");

  extern __shared__ uint4 smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tiles_m = (p.M + BM - 1) / BM;
  const int logical = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tm = logical / tiles_n, tn = logical % tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;

  const bf16_t* Aptr[NA] = {(const bf16_t*)p.A};
  if (DUAL) Aptr[NA - 1] = (const bf16_t*)p.A1;
  const bf16_t* Bt = (const bf16_t*)p.Bt;

  // per-thread source rows (clamped into range; out-of-range rows are masked at the end)
  const bf16_t* a_src[NA][CA];
  const bf16_t* b_src[CB];
  int a_dst[CA], b_dst[CB];
  const int ch = tid & 7;
#pragma unroll
  for (int i = 0; i < CA; ++i) {
    const int row = (tid >> 3) + i * (NT / 8);
    int g = m0 + row;
    g = g < p.M ? g : p.M - 1;
#pragma unroll
    for (int s = 0; s < NA; ++s) a_src[s][i] = Aptr[s] + (int64_t)g * p.lda + ch * 8;
    a_dst[i] = row * 8 + (ch ^ (row & 7));
  }
#pragma unroll
  for (int i = 0; i < CB; ++i) {
    const int row = (tid >> 3) + i * (NT / 8);
    int g = n0 + row;
    g = g < p.N ? g : p.N - 1;
    b_src[i] = Bt + (int64_t)g * p.ldb + ch * 8;
    b_dst[i] = row * 8 + (ch ^ (row & 7));
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint4 ra[NA][CA], rb[CB];
  const int KT = (p.K + 63) >> 6;

  auto load_global = [&](int kt) {
    const int k0 = kt << 6;
    const bool ok = (k0 + ch * 8) < p.K;
#pragma unroll
    for (int s = 0; s < NA; ++s)
#pragma unroll
      for (int i = 0; i < CA; ++i)
        ra[s][i] = ok ? *(const uint4*)(a_src[s][i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < CB; ++i) rb[i] = ok ? *(const uint4*)(b_src[i] + k0) : make_uint4(0, 0, 0, 0);
  };
  auto store_lds = [&](int buf) {
    uint4* sA = smem + buf * STAGE;
    uint4* sB = sA + NA * BM * 8;
#pragma unroll
    for (int s = 0; s < NA; ++s)
#pragma unroll
      for (int i = 0; i < CA; ++i) sA[s * BM * 8 + a_dst[i]] = ra[s][i];
#pragma unroll
    for (int i = 0; i < CB; ++i) sB[b_dst[i]] = rb[i];
  };

  load_global(0);
  store_lds(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) load_global(kt + 1);
    const uint4* sA = smem + cur * STAGE;
    const uint4* sB = sA + NA * BM * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      Frag a[NA][TM], b[TN];
      const int c = ks * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wm * WM + i * 32 + (lane & 31);
#pragma unroll
        for (int s = 0; s < NA; ++s) a[s][i].u = sA[s * BM * 8 + row * 8 + (c ^ (row & 7))];
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int row = wn * WN + j * 32 + (lane & 31);
        b[j].u = sB[row * 8 + (c ^ (row & 7))];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const Frag& af = a[DUAL ? (j & 1) : 0][i];
          if (SWAP)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j].v, af.v, acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, b[j].v, acc[i][j], 0, 0, 0);
        }
    }
    if (kt + 1 < KT) store_lds(cur ^ 1);
    __syncthreads();
  }

  // ---------------------------------------------------------------- epilogue
  constexpr int JSTEP = (ACT == ACT_GLU) ? 2 : 1;
  if (!SCORE) {
    // lane: row = lane & 31; columns 8g + 4(lane>>5) + 0..3 of each 32x32 tile
#pragma unroll
    for (int j = 0; j < TN; j += JSTEP) {
      const int cb = n0 + wn * WN + j * 32;  // GEMM column of this block
      if (cb >= p.N) continue;
      const bool act_here = cb < p.act_cols;
      if (ACT == ACT_GLU && !act_here) {
        // two independent plain blocks
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          const int cbb = cb + jj * 32;
          if (cbb >= p.N) continue;
          const int oc = cbb - p.act_cols / 2;
          char* base;
          int64_t ld;
          int occ;
          if (oc < p.split_col) { base = (char*)p.C0; ld = p.ldc0; occ = oc; }
          else { base = (char*)p.C1; ld = p.ldc1; occ = oc - p.split_col; }
#pragma unroll
          for (int i = 0; i < TM; ++i) {
            const int row = m0 + wm * WM + i * 32 + (lane & 31);
            if (row >= p.M) continue;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              if (cbb + 8 * g + 4 * (lane >> 5) >= p.N) continue;
              const int col = occ + 8 * g + 4 * (lane >> 5);
              const float v0 = acc[i][j + jj][4 * g], v1 = acc[i][j + jj][4 * g + 1];
              const float v2 = acc[i][j + jj][4 * g + 2], v3 = acc[i][j + jj][4 * g + 3];
              if (p.out_f32) *(float4*)(base + ((int64_t)row * ld + col) * 4) = make_float4(v0, v1, v2, v3);
              else *(uint2*)(base + ((int64_t)row * ld + col) * 2) = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
            }
          }
        }
        continue;
      }
      int oc;
      if (ACT == ACT_GLU) oc = cb / 2;
      else oc = cb;
      char* base;
      int64_t ld;
      int occ;
      if (oc < p.split_col) { base = (char*)p.C0; ld = p.ldc0; occ = oc; }
      else { base = (char*)p.C1; ld = p.ldc1; occ = oc - p.split_col; }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = m0 + wm * WM + i * 32 + (lane & 31);
        if (row >= p.M) continue;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          if (ACT != ACT_GLU && cb + 8 * g + 4 * (lane >> 5) >= p.N) continue;
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float z = acc[i][(ACT == ACT_GLU) ? j + 1 : j][4 * g + e];
            const float gt = acc[i][j][4 * g + e];
            v[e] = act_here ? apply_act<ACT>(z, gt) : z;
          }
          const int col = occ + 8 * g + 4 * (lane >> 5);
          if (p.out_f32) *(float4*)(base + ((int64_t)row * ld + col) * 4) = make_float4(v[0], v[1], v[2], v[3]);
          else *(uint2*)(base + ((int64_t)row * ld + col) * 2) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
        }
      }
    }
  } else {
    // lane: column = lane & 31; rows 8g + 4(lane>>5) + 0..3 of each 32x32 tile
    constexpr int BNO = BN / JSTEP;
    float* red2 = (float*)smem;          // [WGM][BNO]
    float* red1 = red2 + WGM * BNO;
#pragma unroll
    for (int j = 0; j < TN; j += JSTEP) {
      float s2 = 0.f, s1 = 0.f;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          const float z = acc[i][(ACT == ACT_GLU) ? j + 1 : j][v];
          const float gt = acc[i][j][v];
          float h = apply_act<ACT>(z, gt);
          h = row < p.M ? h : 0.f;
          s2 += h * h;
          s1 += fabsf(h);
        }
      s2 += __shfl_xor(s2, 32);
      s1 += __shfl_xor(s1, 32);
      if (lane < 32) {
        const int cl = (wn * WN + j * 32) / JSTEP + lane;
        red2[wm * BNO + cl] = s2;
        red1[wm * BNO + cl] = s1;
      }
    }
    __syncthreads();
    for (int t = tid; t < BNO; t += NT) {
      const int col = n0 / JSTEP + t;
      if (col < p.n_out) {
        float a2 = 0.f, a1 = 0.f;
#pragma unroll
        for (int w = 0; w < WGM; ++w) { a2 += red2[w * BNO + t]; a1 += red1[w * BNO + t]; }
        p.part_s2[(int64_t)tm * p.n_out + col] = a2;
        p.part_s1[(int64_t)tm * p.n_out + col] = a1;
      }
    }
  }
}

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

  for (int k0 = 0; k0 < p.K; k0 += BK) {
    const bool ok = (k0 + lk) < p.K;
    float4 va[NA], vb;
#pragma unroll
    for (int s = 0; s < NA; ++s) va[s] = ok ? *(const float4*)(a_src[s] + k0) : make_float4(0, 0, 0, 0);
    vb = ok ? *(const float4*)(b_src + k0) : make_float4(0, 0, 0, 0);
    __syncthreads();
#pragma unroll
    for (int s = 0; s < NA; ++s) {
      sA[s][lk + 0][lrow] = va[s].x; sA[s][lk + 1][lrow] = va[s].y;
      sA[s][lk + 2][lrow] = va[s].z; sA[s][lk + 3][lrow] = va[s].w;
    }
    sB[lk + 0][lrow] = vb.x; sB[lk + 1][lrow] = vb.y; sB[lk + 2][lrow] = vb.z; sB[lk + 3][lrow] = vb.w;
    __syncthreads();
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
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = m0 + ty + 16 * i;
        if (row >= p.M) continue;
        float v;
        if (ACT == ACT_GLU) v = glu_here ? silu_f(acc[i][j]) * acc[i][(j + 2) & 3] : acc[i][j];
        else if (ACT == ACT_GELU) v = cb < p.act_cols ? gelu_f(acc[i][j]) : acc[i][j];
        else v = acc[i][j];
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

// ------------------------------------------------------------------ host launchers

template <int BM, int BN, int WGM, int WGN, int ACT, bool DUAL, bool SCORE>
static int launch_bf16(const GemmArgs& a, hipStream_t st) {
  constexpr int NA = DUAL ? 2 : 1;
  constexpr size_t lds = (size_t)2 * (NA * BM + BN) * 8 * 16;
  auto kern = gemm_bf16_kernel<BM, BN, WGM, WGN, ACT, DUAL, SCORE>;
  static bool configured = false;  // attribute is per function, set once per process
  if (!configured) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return -1;
    configured = true;
  }
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(WGM * WGN * 64), lds, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int ACT, bool DUAL, bool SCORE>
static int launch_f32(const GemmArgs& a, hipStream_t st) {
  const int tiles = ((a.M + 63) / 64) * ((a.N + 63) / 64);
  hipLaunchKernelGGL((gemm_f32_kernel<ACT, DUAL, SCORE>), dim3(tiles), dim3(256), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int gemm_tile_m(int dtype_bf16) { return dtype_bf16 ? 128 : 64; }

int launch_gemm(const GemmArgs& a, int dtype_bf16, int act, bool score, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0) return 0;
  const bool dual = a.A1 != nullptr;
  if (dtype_bf16) {
    if (score) {
      if (act == ACT_GELU) return launch_bf16<128, 128, 2, 2, ACT_GELU, false, true>(a, st);
      if (act == ACT_GLU) return launch_bf16<128, 128, 2, 2, ACT_GLU, false, true>(a, st);
      return -1;
    }
    if (act == ACT_NONE) return launch_bf16<128, 128, 2, 2, ACT_NONE, false, false>(a, st);
    if (act == ACT_GELU) return launch_bf16<128, 128, 2, 2, ACT_GELU, false, false>(a, st);
    if (act == ACT_GLU && !dual) return launch_bf16<128, 128, 2, 2, ACT_GLU, false, false>(a, st);
    if (act == ACT_GLU && dual) return launch_bf16<128, 128, 2, 2, ACT_GLU, true, false>(a, st);
    return -1;
  }
  if (score) {
    if (act == ACT_GELU) return launch_f32<ACT_GELU, false, true>(a, st);
    if (act == ACT_GLU) return launch_f32<ACT_GLU, false, true>(a, st);
    return -1;
  }
  if (act == ACT_NONE) return launch_f32<ACT_NONE, false, false>(a, st);
  if (act == ACT_GELU) return launch_f32<ACT_GELU, false, false>(a, st);
  if (act == ACT_GLU && !dual) return launch_f32<ACT_GLU, false, false>(a, st);
  if (act == ACT_GLU && dual) return launch_f32<ACT_GLU, true, false>(a, st);
  return -1;
}

}  // namespace ffs
