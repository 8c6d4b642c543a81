// Rank-r factors of the remainder matrices, computed on the device so that a split can be
// built without a host factorisation (Sec. 4.2 / 5.1.1: a low-rank decomposition of U2 and V2,
// each on its own).  Instead of a full SVD: the randomised range finder of Halko, Martinsson
// and Tropp (2011, Alg. 4.1) on the d_model side of every matrix,
//     Z [d, m] (W1[:, rest], Wg[:, rest] or W2[rest, :]^T),  Y^T = Omega Z^T  [r, d],
//     B^T = orthonormal rows spanning the rows of Y^T,       C = B^T Z  [r, m],
// so that Z ~= B C.  Omega [r, m] is a counter-based Rademacher matrix (the same signs on any
// machine).  The rows of Y^T are orthonormalised with the Newton-Schulz iteration for the
// polar factor, X <- (1.5 I - 0.5 X X^T) X from X = Y^T / ||Y||_F, because it consists of
// products only: everything here runs on the fp32 GEMM of gemm.hip plus a few elementwise
// kernels, in fp32, whatever the storage type of the weights.
#include "factor.h"
#include <math.h>

namespace ffsplit {

namespace {

__device__ __forceinline__ uint32_t fmix32(uint32_t h) {   // finaliser of the public MurmurHash3
  h ^= h >> 16; h *= 0x85EBCA6Bu; h ^= h >> 13; h *= 0xC2B2AE35u; h ^= h >> 16;
  return h;
}

template <typename T>
__device__ __forceinline__ float ldf(const T* p, int64_t i);
template <>
__device__ __forceinline__ float ldf<float>(const float* p, int64_t i) { return p[i]; }
template <>
__device__ __forceinline__ float ldf<bf16_t>(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }

// Z [d, m4] and Zt [m4, d] (fp32, zero in the padding columns) from the weights:
// down = 0: Z[c][j] = W[c][rest[j]] (W [d, d_ff]);  down = 1: Z[c][j] = W[rest[j]][c] (W [d_ff, d])
template <typename T>
__global__ void gather_z_kernel(const T* W, int d, int d_ff, const int32_t* rest, int m, int m4, int down, float* Z,
                                float* Zt) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)d * m4) return;
  const int c = (int)(id / m4), j = (int)(id % m4);
  float v = 0.f;
  if (j < m) {
    const int n = rest[j];
    v = down ? ldf<T>(W, (int64_t)n * d + c) : ldf<T>(W, (int64_t)c * d_ff + n);
  }
  Z[id] = v;
  Zt[(int64_t)j * d + c] = v;
}

// Omega [r4, m4]: entry (i, j) = +-1 from the top bit of fmix32(index * 0x9E3779B1 + key),
// index = i * m + j; zero in the padding
__global__ void rademacher_kernel(float* Om, int r, int m, int r4, int m4, uint32_t key) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)r4 * m4) return;
  const int i = (int)(id / m4), j = (int)(id % m4);
  float v = 0.f;
  if (i < r && j < m) {
    const uint32_t h = fmix32((uint32_t)(i * m + j) * 0x9E3779B1u + key);
    v = (h >> 31) ? -1.f : 1.f;
  }
  Om[id] = v;
}

// sum of squares in two fixed-order stages: 256 block partials, then one block
__global__ void __launch_bounds__(256) sumsq_stage1_kernel(const float* x, int64_t n, float* part) {
  __shared__ float red[256];
  float s = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)256 * gridDim.x) s += x[i] * x[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}
__global__ void __launch_bounds__(256) sumsq_stage2_kernel(float* part, int n_part) {
  __shared__ float red[256];
  red[threadIdx.x] = (int)threadIdx.x < n_part ? part[threadIdx.x] : 0.f;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) part[256] = red[0] > 0.f ? 1.0f / sqrtf(red[0]) : 0.f;   // scale for the next kernel
}
__global__ void scale_kernel(float* x, int64_t n, const float* scale) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id < n) x[id] *= scale[0];
}

// S <- 1.5 I - 0.5 S  (n x n)
__global__ void ns_update_kernel(float* S, int n) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)n * n) return;
  const int i = (int)(id / n), j = (int)(id % n);
  S[id] = (i == j ? 1.5f : 0.f) - 0.5f * S[id];
}

// dst[a][b] = src[b][a] (fp32), a < rows_dst, b < cols_dst
__global__ void transpose_f32_kernel(const float* src, int64_t lds, float* dst, int64_t ldd, int rows_dst, int cols_dst) {
  __shared__ float tile[32][33];
  const int a0 = blockIdx.y * 32, b0 = blockIdx.x * 32;
  for (int i = threadIdx.y; i < 32; i += 8) {
    const int b = b0 + i, a = a0 + threadIdx.x;
    tile[i][threadIdx.x] = (b < cols_dst && a < rows_dst) ? src[(int64_t)b * lds + a] : 0.f;
  }
  __syncthreads();
  for (int i = threadIdx.y; i < 32; i += 8) {
    const int a = a0 + i, b = b0 + threadIdx.x;
    if (a < rows_dst && b < cols_dst) dst[(int64_t)a * ldd + b] = tile[threadIdx.x][i];
  }
}

// dst [rows, cols] (bf16 or fp32, contiguous) = src[a][b] or src[b][a]
template <typename T>
__global__ void emit_kernel(const float* src, int64_t lds, int transposed, T* dst, int rows, int cols) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)rows * cols) return;
  const int a = (int)(id / cols), b = (int)(id % cols);
  const float v = transposed ? src[(int64_t)b * lds + a] : src[(int64_t)a * lds + b];
  if constexpr (sizeof(T) == 4) dst[id] = v;
  else dst[id] = (T)(pack_bf16x2(v, 0.f) & 0xffffu);
}

struct FactorWs {
  size_t off_z, off_zt, off_om, off_xa, off_xb, off_xt, off_s, off_sp, off_c, off_red, total;
  int m4, r4;
  int s_split;   // split of the reduction of the Gram product X X^T (r x r, few tiles, long K)
};

FactorWs make_factor_ws(const ffsplit_desc_t& d) {
  FactorWs w = {};
  const int m = d.d_ff - d.k;
  w.m4 = round_up(m > 0 ? m : 4, 4);
  w.r4 = round_up(d.rank > 0 ? d.rank : 4, 4);
  size_t off = 0;
  const size_t dm = (size_t)d.d_model;
  w.off_z = off; off = align256(off + dm * w.m4 * 4);
  w.off_zt = off; off = align256(off + dm * w.m4 * 4);
  w.off_om = off; off = align256(off + (size_t)w.r4 * w.m4 * 4);
  w.off_xa = off; off = align256(off + (size_t)w.r4 * dm * 4);
  w.off_xb = off; off = align256(off + (size_t)w.r4 * dm * 4);
  w.off_xt = off; off = align256(off + (size_t)w.r4 * dm * 4);
  w.off_s = off; off = align256(off + (size_t)w.r4 * w.r4 * 4);
  // The Gram product has (r / 64)^2 tiles of 64 x 64 and K = d_model: split it so that a few
  // hundred workgroups exist, at least 16 slabs of 16 each (the partial sums need whole
  // 8-column chunks).
  {
    const int tiles = ((w.r4 + 63) / 64) * ((w.r4 + 63) / 64);
    int sp = 512 / (tiles > 0 ? tiles : 1);
    if (sp > (int)dm / 256) sp = (int)dm / 256;
    if (sp > 16) sp = 16;
    if (sp < 1 || (w.r4 & 7)) sp = 1;
    w.s_split = sp;
  }
  w.off_sp = off; if (w.s_split > 1) off = align256(off + (size_t)w.s_split * w.r4 * w.r4 * 4);
  w.off_c = off; off = align256(off + (size_t)w.r4 * w.m4 * 4);
  w.off_red = off; off = align256(off + 260 * 4);
  w.total = off;
  return w;
}

int gemm_nt(const float* A, int64_t lda, const float* Bt, int64_t ldb, int M, int N, int K, float* C, int64_t ldc,
            hipStream_t st) {
  GemmArgs g = {};
  g.A = A; g.lda = lda; g.Bt = Bt; g.ldb = ldb; g.M = M; g.N = N; g.K = K;
  g.split_col = N; g.C0 = C; g.ldc0 = ldc; g.n_store = N;
  return launch_gemm_f32(g, ACT_NONE, false, st);
}

#define FK(expr)                 \
  do {                           \
    if ((expr) != 0) return -1;  \
  } while (0)
#define FKL()                                        \
  do {                                               \
    if (hipGetLastError() != hipSuccess) return -1;  \
  } while (0)

}  // namespace

size_t factorize_ws_bytes(const ffsplit_desc_t& d) { return make_factor_ws(d).total; }

int launch_factorize(const ffsplit_desc_t& d, const void* W1, const void* Wg, const void* W2, const int32_t* rest,
                     uint32_t seed, void* const* factors, char* ws, hipStream_t st) {
  const int dm = d.d_model, m = d.d_ff - d.k, r = d.rank;
  if (m <= 0 || r <= 0) return 0;
  const FactorWs w = make_factor_ws(d);
  const int m4 = w.m4, r4 = w.r4;
  float* Z = (float*)(ws + w.off_z); float* Zt = (float*)(ws + w.off_zt); float* Om = (float*)(ws + w.off_om);
  float* Xa = (float*)(ws + w.off_xa); float* Xb = (float*)(ws + w.off_xb); float* Xt = (float*)(ws + w.off_xt);
  float* S = (float*)(ws + w.off_s); float* C = (float*)(ws + w.off_c); float* red = (float*)(ws + w.off_red);
  float* Sp = (float*)(ws + w.off_sp);
  const bool bf = d.dtype == FFSPLIT_BF16;
  // Steps of x <- 1.5 x - 0.5 x^3: a singular value far below 1 grows by 1.5 per step, then
  // converges quadratically (about ten more steps to fp32 accuracy).  Budget: singular values
  // down to 1 / (64 r) of the Frobenius norm (a square Gaussian Y, r = d_model, has its smallest
  // near r^-1.5 of it); a basis direction below that comes out shorter than unit length.
  const int n_iter = 10 + (int)ceil(log(64.0 * (double)r) / log(1.5));
  const void* Ws[3] = {W1, Wg, W2};
  for (int which = 0; which < 3; ++which) {
    if (which == 1 && d.act != FFSPLIT_ACT_SWIGLU) continue;
    const int down = which == 2;
    const int64_t nz = (int64_t)dm * m4;
    const unsigned gz = (unsigned)((nz + 255) / 256);
    if (bf) hipLaunchKernelGGL(gather_z_kernel<bf16_t>, dim3(gz), dim3(256), 0, st, (const bf16_t*)Ws[which], dm, d.d_ff, rest, m, m4, down, Z, Zt);
    else hipLaunchKernelGGL(gather_z_kernel<float>, dim3(gz), dim3(256), 0, st, (const float*)Ws[which], dm, d.d_ff, rest, m, m4, down, Z, Zt);
    FKL();
    uint32_t key = seed + 0x9E3779B9u * (uint32_t)which;
    key ^= key >> 16; key *= 0x85EBCA6Bu; key ^= key >> 13; key *= 0xC2B2AE35u; key ^= key >> 16;
    const int64_t no = (int64_t)r4 * m4;
    hipLaunchKernelGGL(rademacher_kernel, dim3((unsigned)((no + 255) / 256)), dim3(256), 0, st, Om, r, m, r4, m4, key);
    FKL();
    // Y^T = Omega Z^T, scaled to unit Frobenius norm
    FK(gemm_nt(Om, m4, Z, m4, r4, dm, m4, Xa, dm, st));
    const int64_t nx = (int64_t)r4 * dm;
    hipLaunchKernelGGL(sumsq_stage1_kernel, dim3(256), dim3(256), 0, st, Xa, nx, red);
    hipLaunchKernelGGL(sumsq_stage2_kernel, dim3(1), dim3(256), 0, st, red, 256);
    hipLaunchKernelGGL(scale_kernel, dim3((unsigned)((nx + 255) / 256)), dim3(256), 0, st, Xa, nx, red + 256);
    FKL();
    float* X = Xa; float* Xn = Xb;
    for (int it = 0; it < n_iter; ++it) {
      if (w.s_split > 1) {
        GemmArgs g = {};
        g.A = X; g.lda = dm; g.Bt = X; g.ldb = dm; g.M = r4; g.N = r4; g.K = dm;
        g.split_col = r4; g.C0 = Sp; g.ldc0 = r4; g.n_store = r4; g.partial = 1;
        FK(launch_gemm_f32(g, ACT_NONE, false, st, w.s_split));
        FK(launch_splitk_reduce(Sp, w.s_split, r4, r4, r4, S, r4, 0, st, 1));
      } else {
        FK(gemm_nt(X, dm, X, dm, r4, r4, dm, S, r4, st));
      }
      hipLaunchKernelGGL(ns_update_kernel, dim3((unsigned)(((int64_t)r4 * r4 + 255) / 256)), dim3(256), 0, st, S, r4);
      hipLaunchKernelGGL(transpose_f32_kernel, dim3((r4 + 31) / 32, (dm + 31) / 32), dim3(32, 8), 0, st, X, (int64_t)dm, Xt,
                         (int64_t)r4, dm, r4);
      FKL();
      FK(gemm_nt(S, r4, Xt, r4, r4, dm, r4, Xn, dm, st));
      float* t = X; X = Xn; Xn = t;
    }
    // C = B^T Z
    FK(gemm_nt(X, dm, Zt, dm, r4, m4, dm, C, m4, st));
    // factors in the caller's convention and type
    void* Pf = factors[which == 0 ? 0 : (which == 1 ? 2 : 4)];
    void* Qf = factors[which == 0 ? 1 : (which == 1 ? 3 : 5)];
    const float* psrc = down ? C : X;      // P = B [d, r] (up, gate) or C^T [m, r] (down)
    const float* qsrc = down ? X : C;      // Q = C [r, m] (up, gate) or B^T [r, d] (down)
    const int prow = down ? m : dm, qcol = down ? dm : m;
    const int64_t pld = down ? m4 : dm, qld = down ? dm : m4;
    const int64_t np_ = (int64_t)prow * r, nq = (int64_t)r * qcol;
    if (bf) {
      hipLaunchKernelGGL(emit_kernel<bf16_t>, dim3((unsigned)((np_ + 255) / 256)), dim3(256), 0, st, psrc, pld, 1, (bf16_t*)Pf, prow, r);
      hipLaunchKernelGGL(emit_kernel<bf16_t>, dim3((unsigned)((nq + 255) / 256)), dim3(256), 0, st, qsrc, qld, 0, (bf16_t*)Qf, r, qcol);
    } else {
      hipLaunchKernelGGL(emit_kernel<float>, dim3((unsigned)((np_ + 255) / 256)), dim3(256), 0, st, psrc, pld, 1, (float*)Pf, prow, r);
      hipLaunchKernelGGL(emit_kernel<float>, dim3((unsigned)((nq + 255) / 256)), dim3(256), 0, st, qsrc, qld, 0, (float*)Qf, r, qcol);
    }
    FKL();
  }
  return 0;
}

}  // namespace ffsplit
