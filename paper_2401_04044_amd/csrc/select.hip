// Bit-exact top-k of the neuron scores (heavy-hitter selection, Sec. 4.1/5.1.1).
// Integer work only: scores are mapped to order-preserving uint32 keys, the k-th
// largest key is found by a 4-pass radix select, the chosen elements are
// compacted in index order (equal keys: lowest indices first) and finally ranked
// by counting, which yields the order (score descending, index ascending).
#include "prep.h"

namespace ffsplit {

__device__ __forceinline__ uint32_t score_key(float s, int* saw_nan) {
  uint32_t b = __float_as_uint(s);
  if ((b & 0x7fffffffu) > 0x7f800000u) { *saw_nan = 1; return 0xffffffffu; }
  if (b == 0x80000000u) b = 0u;                       // -0 counts as +0
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);  // monotone in the float order
}

__global__ void __launch_bounds__(1024) select_compact_kernel(const float* scores, int n, int k, uint32_t* keys,
                                                              uint32_t* cand_key, int32_t* cand_idx, int32_t* perm,
                                                              int32_t* nan_flag) {
  __shared__ int hist[256];
  __shared__ int wsum[16];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need, s_nan;
  const int tid = threadIdx.x;
  if (tid == 0) { s_nan = 0; s_prefix = 0; s_need = k; }
  __syncthreads();
  int saw = 0;
  for (int i = tid; i < n; i += 1024) keys[i] = score_key(scores[i], &saw);
  if (saw) s_nan = 1;
  __syncthreads();
  if (tid == 0 && nan_flag) *nan_flag = s_nan ? -7 : 0;
  if (k <= 0) {
    if (perm) for (int i = tid; i < n; i += 1024) perm[i] = i;
    return;
  }
  // radix select, most significant byte first
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = s_prefix;
    for (int i = tid; i < n; i += 1024) {
      const uint32_t key = keys[i];
      const bool match = pass == 0 ? true : ((key >> (shift + 8)) == prefix);
      if (match) atomicAdd(&hist[(key >> shift) & 255], 1);
    }
    __syncthreads();
    if (tid == 0) {
      int need = s_need, cum = 0, b = 255;
      for (; b > 0; --b) {
        if (cum + hist[b] >= need) break;
        cum += hist[b];
      }
      s_need = need - cum;
      s_prefix = (prefix << 8) | (uint32_t)b;
    }
    __syncthreads();
  }
  const uint32_t thr = s_prefix;
  const int need = s_need;  // how many keys equal to thr are taken (lowest indices)
  int eq_base = 0, sel_base = 0, rest_base = 0;
  for (int base = 0; base < n; base += 1024) {
    const int i = base + tid;
    const bool in = i < n;
    const uint32_t key = in ? keys[i] : 0u;
    const bool eq = in && key == thr;
    int tot;
    const int eq_rank = eq_base + block_prefix_1024(eq, wsum, &tot);
    eq_base += tot;
    const bool sel = in && (key > thr || (eq && eq_rank < need));
    const int pos = sel_base + block_prefix_1024(sel, wsum, &tot);
    sel_base += tot;
    const bool rest = in && !sel;
    const int rpos = rest_base + block_prefix_1024(rest, wsum, &tot);
    rest_base += tot;
    if (sel) { cand_key[pos] = key; cand_idx[pos] = i; }
    if (rest && perm) perm[k + rpos] = i;
  }
}

// rank of candidate a = #(keys greater) + #(equal keys at an earlier position)
__global__ void __launch_bounds__(256) select_rank_kernel(const uint32_t* cand_key, const int32_t* cand_idx, int k,
                                                          int32_t* idx, int32_t* perm) {
  __shared__ uint32_t tile[256];
  const int a = blockIdx.x * 256 + threadIdx.x;
  const uint32_t ka = a < k ? cand_key[a] : 0u;
  int rank = 0;
  for (int b0 = 0; b0 < k; b0 += 256) {
    __syncthreads();
    tile[threadIdx.x] = (b0 + threadIdx.x) < k ? cand_key[b0 + threadIdx.x] : 0u;
    __syncthreads();
    const int lim = min(256, k - b0);
    for (int b = 0; b < lim; ++b) {
      const uint32_t kb = tile[b];
      rank += (kb > ka) || (kb == ka && (b0 + b) < a);
    }
  }
  if (a < k) {
    const int32_t v = cand_idx[a];
    idx[rank] = v;
    if (perm) perm[rank] = v;
  }
}

size_t select_workspace_bytes(int d_ff) { return (size_t)12 * (size_t)(d_ff > 0 ? d_ff : 1) + 256; }

int launch_select(const float* scores, int d_ff, int k, int32_t* idx, int32_t* perm, int32_t* nan_flag, void* ws,
                  hipStream_t st) {
  if (d_ff <= 0) return 0;
  uint32_t* keys = (uint32_t*)ws;
  uint32_t* cand_key = keys + d_ff;
  int32_t* cand_idx = (int32_t*)(cand_key + d_ff);
  hipLaunchKernelGGL(select_compact_kernel, dim3(1), dim3(1024), 0, st, scores, d_ff, k, keys, cand_key, cand_idx,
                     perm, nan_flag);
  if (hipGetLastError() != hipSuccess) return -1;
  if (k > 0) {
    hipLaunchKernelGGL(select_rank_kernel, dim3((k + 255) / 256), dim3(256), 0, st, cand_key, cand_idx, k, idx, perm);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

}  // namespace ffsplit
