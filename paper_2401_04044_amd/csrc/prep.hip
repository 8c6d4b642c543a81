// One-off and small kernels around the GEMMs: zero fill, permuted transposes
// (neuron gather + packing of Eq. 2's partition), the fixed-order reduction of
// the score partials and the W2 row-norm / score finalisation of Eq. 3.
#include "prep.h"

namespace ffsplit {

__global__ void fill_zero_kernel(uint4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

int launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return 0;
  const size_t n16 = bytes / 16;  // callers keep sizes a multiple of 16
  int blocks = (int)((n16 + 255) / 256);
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, (uint4*)p, n16);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// dst[f(n)][coff + c] = src[cmap(c)][nmap(n)],  n < n_count, c < c_count.
template <typename T>
__global__ void permute_transpose_kernel(const PermArgs a) {
  __shared__ T tile[32][33];
  const int n0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
  const int tx = threadIdx.x, ty = threadIdx.y;
  const T* src = (const T*)a.src;
  T* dst = (T*)a.dst;
  const int n = n0 + tx;
  int64_t scol = -1;
  if (n < a.n_count) scol = a.nmap ? a.nmap[a.nmap_off + n] : n;
  for (int cc = ty; cc < 32; cc += 8) {
    const int c = c0 + cc;
    T v = 0;
    if (c < a.c_count && scol >= 0) {
      const int64_t srow = a.cmap ? a.cmap[a.cmap_off + c] : c;
      v = src[srow * a.lds + scol];
    }
    tile[cc][tx] = v;
  }
  __syncthreads();
  const int c = c0 + tx;
  for (int nn = ty; nn < 32; nn += 8) {
    const int nq = n0 + nn;
    if (nq < a.n_count && c < a.c_count) {
      int64_t drow;
      if (a.glu_mode == 0) drow = a.row_off + nq;
      else drow = a.row_off + (int64_t)(nq >> 5) * 64 + (nq & 31) + (a.glu_mode == 2 ? 32 : 0);
      const int64_t dcol = a.coff + c;
      if (a.dst_tiled)
        dst[((drow >> 5) * (a.ldd >> 4) + (dcol >> 4)) * 512 + ((dcol >> 3) & 1) * 256 + (drow & 31) * 8 + (dcol & 7)] =
            tile[tx][nn];
      else
        dst[drow * a.ldd + dcol] = tile[tx][nn];
    }
  }
}

int launch_permute_transpose(const PermArgs& a, int esize, hipStream_t st) {
  if (a.n_count <= 0 || a.c_count <= 0) return 0;
  dim3 grid((a.n_count + 31) / 32, (a.c_count + 31) / 32), block(32, 8);
  if (esize == 2) hipLaunchKernelGGL(permute_transpose_kernel<uint16_t>, grid, block, 0, st, a);
  else hipLaunchKernelGGL(permute_transpose_kernel<uint32_t>, grid, block, 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// acc[j] += sum_t part_s2[t][j] ; acc[d_ff + j] += sum_t part_s1[t][j]  (t ascending)
__global__ void reduce_partials_kernel(const float* part_s2, const float* part_s1, int tiles, int n_out,
                                       int d_ff, float* acc) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d_ff) return;
  float s2 = 0.f, s1 = 0.f;
  for (int t = 0; t < tiles; ++t) {
    s2 += part_s2[(int64_t)t * n_out + j];
    s1 += part_s1[(int64_t)t * n_out + j];
  }
  acc[j] += s2;
  acc[d_ff + j] += s1;
}

int launch_reduce_partials(const float* p2, const float* p1, int tiles, int n_out, int d_ff, float* acc,
                           hipStream_t st) {
  if (d_ff <= 0) return 0;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((d_ff + 255) / 256), dim3(256), 0, st, p2, p1, tiles, n_out,
                     d_ff, acc);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// One wavefront per neuron: n2 = sum_c W2[j,c]^2 by lane-strided partial sums
// and a fixed butterfly of wavefront shuffles, then the score of the given kind.
template <bool BF16>
__global__ void finalize_scores_kernel(const void* W2, int d_model, int d_ff, const float* acc, float t_total,
                                       int kind, float* scores) {
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (j >= d_ff) return;
  float n2 = 0.f;
  if (kind != 2) {
    if (BF16) {
      const bf16_t* row = (const bf16_t*)W2 + (int64_t)j * d_model;
      for (int c = lane * 8; c < d_model; c += 64 * 8) {
        const uint4 v = *(const uint4*)(row + c);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = __uint_as_float(w[e] << 16), hi = __uint_as_float(w[e] & 0xffff0000u);
          n2 = fmaf(lo, lo, n2);
          n2 = fmaf(hi, hi, n2);
        }
      }
    } else {
      const float* row = (const float*)W2 + (int64_t)j * d_model;
      for (int c = lane * 4; c < d_model; c += 64 * 4) {
        const float4 v = *(const float4*)(row + c);
        n2 = fmaf(v.x, v.x, n2); n2 = fmaf(v.y, v.y, n2); n2 = fmaf(v.z, v.z, n2); n2 = fmaf(v.w, v.w, n2);
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) n2 += __shfl_xor(n2, o);
  }
  if (lane == 0) {
    float s;
    if (kind == 0) s = acc[j] * n2;
    else if (kind == 1) s = (acc[d_ff + j] / fmaxf(t_total, 1.f)) * sqrtf(n2);
    else s = acc[j];
    scores[j] = s + 0.f;
  }
}

int launch_finalize_scores(const void* W2, int bf16, int d_model, int d_ff, const float* acc, float t_total,
                           int kind, float* scores, hipStream_t st) {
  if (d_ff <= 0) return 0;
  const int blocks = (d_ff + 3) / 4;
  if (bf16) hipLaunchKernelGGL(finalize_scores_kernel<true>, dim3(blocks), dim3(256), 0, st, W2, d_model, d_ff, acc, t_total, kind, scores);
  else hipLaunchKernelGGL(finalize_scores_kernel<false>, dim3(blocks), dim3(256), 0, st, W2, d_model, d_ff, acc, t_total, kind, scores);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ------------------------------------------------------------------ stack harness kernels

// out[t, :] = x[t, :] / sqrt(mean(x[t, :]^2) + eps), one workgroup per token, fp32 sums added in
// a fixed order (lane-strided partials, wavefront butterfly, then the four wavefronts in order).
template <bool BF16>
__global__ void __launch_bounds__(256) token_rmsnorm_kernel(const float* x, int d, float eps, void* out) {
  __shared__ float wsum[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* row = x + (int64_t)blockIdx.x * d;
  // rows of up to 8192 elements stay in registers between the sum and the scaling (one read
  // of the stream); longer rows are read a second time
  constexpr int NV = 8;
  float4 v[NV];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = tid * 4 + i * 1024;
    v[i] = c < d ? *(const float4*)(row + c) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    s = fmaf(v[i].x, v[i].x, s); s = fmaf(v[i].y, v[i].y, s); s = fmaf(v[i].z, v[i].z, s); s = fmaf(v[i].w, v[i].w, s);
  }
  for (int c = tid * 4 + NV * 1024; c < d; c += 1024) {
    const float4 w = *(const float4*)(row + c);
    s = fmaf(w.x, w.x, s); s = fmaf(w.y, w.y, s); s = fmaf(w.z, w.z, s); s = fmaf(w.w, w.w, s);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
  if (lane == 0) wsum[wave] = s;
  __syncthreads();
  const float tot = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  auto emit = [&](int c, const float4& w) {
    if (BF16) {
      *(uint2*)((bf16_t*)out + (int64_t)blockIdx.x * d + c) =
          make_uint2(pack_bf16x2(w.x * inv, w.y * inv), pack_bf16x2(w.z * inv, w.w * inv));
    } else {
      *(float4*)((float*)out + (int64_t)blockIdx.x * d + c) = make_float4(w.x * inv, w.y * inv, w.z * inv, w.w * inv);
    }
  };
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = tid * 4 + i * 1024;
    if (c < d) emit(c, v[i]);
  }
  for (int c = tid * 4 + NV * 1024; c < d; c += 1024) emit(c, *(const float4*)(row + c));
}

int launch_token_rmsnorm(const float* x, int64_t T, int d, float eps, int bf16, void* out, hipStream_t st) {
  if (T <= 0) return 0;
  if (bf16) hipLaunchKernelGGL(token_rmsnorm_kernel<true>, dim3((unsigned)T), dim3(256), 0, st, x, d, eps, out);
  else hipLaunchKernelGGL(token_rmsnorm_kernel<false>, dim3((unsigned)T), dim3(256), 0, st, x, d, eps, out);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// packed[i] = b1[idx[i]] for i < k, 0 up to kp; packed[kp + i] = b1[rest[i]] for i < m, 0 up to kp + mp
template <typename T>
__global__ void pack_neuron_bias_kernel(const T* b1, const int32_t* idx, const int32_t* rest, int k, int kp, int m,
                                        int mp, float* out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= kp + mp) return;
  int src = -1;
  if (i < k) src = idx[i];
  else if (i >= kp && i - kp < m) src = rest[i - kp];
  float v = 0.f;
  if (src >= 0) {
    if (sizeof(T) == 2) v = bf16_to_f32((bf16_t)b1[src]);
    else v = __uint_as_float((uint32_t)b1[src]);
  }
  out[i] = v;
}

int launch_pack_neuron_bias(const void* b1, int bf16, const int32_t* idx, const int32_t* rest, int k, int kp, int m,
                            int mp, float* out, hipStream_t st) {
  const int n = kp + mp;
  if (n <= 0) return 0;
  if (bf16) hipLaunchKernelGGL(pack_neuron_bias_kernel<uint16_t>, dim3((n + 255) / 256), dim3(256), 0, st,
                               (const uint16_t*)b1, idx, rest, k, kp, m, mp, out);
  else hipLaunchKernelGGL(pack_neuron_bias_kernel<uint32_t>, dim3((n + 255) / 256), dim3(256), 0, st,
                          (const uint32_t*)b1, idx, rest, k, kp, m, mp, out);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace ffsplit
