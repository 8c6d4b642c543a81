// Bit-exact top-k of the neuron scores (heavy-hitter selection, Sec. 4.1/5.1.1).
// Integer work only: scores are mapped to order-preserving uint32 keys, the k-th
// largest key is found by a 32-step search over its bits (each step one count over the
// keys, which a workgroup of 1024 threads holds in registers), the chosen elements are
// compacted in index order (equal keys: lowest indices first) and finally ranked
// by counting, which yields the order (score descending, index ascending).
#include "prep.h"
#include <atomic>

namespace ffsplit {

// Scratch of the entry point that allocates nothing (ffsplit_select_heavy_static): one copy per
// GPU the library runs on, held until the process ends.  In host code this name is only a
// stand-in for the symbol; the device address comes from hipGetSymbolAddress (below).
constexpr int SELECT_STATIC_MAX_DFF = 65536;
constexpr size_t SELECT_STATIC_BYTES = (size_t)12 * SELECT_STATIC_MAX_DFF + 256;
static __device__ __align__(256) unsigned char scratch[SELECT_STATIC_BYTES];

__device__ __forceinline__ uint32_t score_key(float s, int* saw_nan) {
  uint32_t b = __float_as_uint(s);
  if ((b & 0x7fffffffu) > 0x7f800000u) { *saw_nan = 1; return 0xffffffffu; }
  if (b == 0x80000000u) b = 0u;                       // -0 counts as +0
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);  // monotone in the float order
}

// Exclusive prefix sum of v over the 1024 threads of a block, in thread order.  wsum: 16 ints
// of LDS.  Every thread must call it.
__device__ __forceinline__ int block_scan_1024(int v, int* wsum) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < 16; ++w) before += w < wave ? wsum[w] : 0;
  return before + inc - v;
}

template <int KPT>
__global__ void __launch_bounds__(1024) select_compact_kernel(const float* scores, int n, int k, uint32_t* keys,
                                                              uint32_t* cand_key, int32_t* cand_idx, int32_t* perm,
                                                              int32_t* nan_flag) {
  __shared__ int wsum[16];
  __shared__ int csum[2][16];
  __shared__ int s_nan;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) s_nan = 0;
  __syncthreads();
  // every thread owns a contiguous run of elements; the first KPT keys of the run stay in
  // registers (key 0 = no element: real keys are > 0), longer runs continue in `keys`
  const int run = (n + 1023) / 1024;
  const int i0 = min(n, tid * run), i1 = min(n, i0 + run);
  uint32_t kreg[KPT];
  int saw = 0;
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const int i = i0 + j;
    kreg[j] = (j < run && i < i1) ? score_key(scores[i], &saw) : 0u;
  }
  for (int i = i0 + KPT; i < i1; ++i) keys[i] = score_key(scores[i], &saw);
  if (saw) s_nan = 1;
  __syncthreads();
  if (tid == 0 && nan_flag) *nan_flag = s_nan ? -7 : 0;
  if (k <= 0) {
    if (perm) for (int i = tid; i < n; i += 1024) perm[i] = i;
    return;
  }
  // number of keys >= c (c > 0), the same value in every thread; buf alternates so that one
  // barrier per call is enough
  int buf = 0;
  auto count_ge = [&](uint32_t c) -> int {
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) cnt += kreg[j] >= c;
    for (int i = i0 + KPT; i < i1; ++i) cnt += keys[i] >= c;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
    if (lane == 0) csum[buf][wave] = cnt;
    __syncthreads();
    int tot = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += csum[buf][w];
    buf ^= 1;
    return tot;
  };
  // the k-th largest key, bit by bit from the top: the largest P with at least k keys >= P
  uint32_t thr = 0u;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t c = thr | (1u << bit);
    if (count_ge(c) >= k) thr = c;
  }
  const int above = thr == 0xffffffffu ? 0 : count_ge(thr + 1u);
  const int need = k - above;  // how many keys equal to thr are taken (lowest indices)
  // Compaction in index order over the threads' runs: two block scans (equal keys, then
  // selected elements).
  int eq_cnt = 0;
#pragma unroll
  for (int j = 0; j < KPT; ++j) eq_cnt += kreg[j] == thr;     // thr > 0: empty slots never match
  for (int i = i0 + KPT; i < i1; ++i) eq_cnt += keys[i] == thr;
  int eq_before = block_scan_1024(eq_cnt, wsum);
  int sel_cnt = 0;
  {
    int e = eq_before;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const bool eq = kreg[j] == thr;
      sel_cnt += kreg[j] > thr || (eq && e < need);
      e += eq;
    }
    for (int i = i0 + KPT; i < i1; ++i) {
      const uint32_t key = keys[i];
      const bool eq = key == thr;
      sel_cnt += key > thr || (eq && e < need);
      e += eq;
    }
  }
  int sp = block_scan_1024(sel_cnt, wsum);   // selected elements before this thread's run
  auto place = [&](uint32_t key, int i) {
    const bool eq = key == thr;
    const bool sel = key > thr || (eq && eq_before < need);
    eq_before += eq;
    if (sel) { cand_key[sp] = key; cand_idx[sp] = i; ++sp; }
    else if (perm) perm[k + (i - sp)] = i;     // i - sp = elements before i that were not selected
  };
#pragma unroll
  for (int j = 0; j < KPT; ++j)
    if (i0 + j < i1 && j < run) place(kreg[j], i0 + j);
  for (int i = i0 + KPT; i < i1; ++i) place(keys[i], i);
}

// rank of candidate a = #(keys greater) + #(equal keys at an earlier position); one wavefront
// per candidate, the lanes share the comparisons
__global__ void __launch_bounds__(256) select_rank_kernel(const uint32_t* cand_key, const int32_t* cand_idx, int k,
                                                          int32_t* idx, int32_t* perm) {
  const int a = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (a >= k) return;
  const uint32_t ka = cand_key[a];
  int rank = 0;
  for (int b = lane; b < k; b += 64) {
    const uint32_t kb = cand_key[b];
    rank += (kb > ka) || (kb == ka && b < a);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) rank += __shfl_xor(rank, o);
  if (lane == 0) {
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
  // registers for the whole run where it is short (the search makes 33 passes over them)
  if (d_ff <= 8 * 1024)
    hipLaunchKernelGGL(select_compact_kernel<8>, dim3(1), dim3(1024), 0, st, scores, d_ff, k, keys, cand_key,
                       cand_idx, perm, nan_flag);
  else
    hipLaunchKernelGGL(select_compact_kernel<32>, dim3(1), dim3(1024), 0, st, scores, d_ff, k, keys, cand_key,
                       cand_idx, perm, nan_flag);
  if (hipGetLastError() != hipSuccess) return -1;
  if (k > 0) {
    hipLaunchKernelGGL(select_rank_kernel, dim3((k + 3) / 4), dim3(256), 0, st, cand_key, cand_idx, k, idx, perm);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

int select_static_max_dff() { return SELECT_STATIC_MAX_DFF; }

// Device address of this GPU's copy of `scratch`, looked up once per device (with that device
// current) and kept; nullptr on failure.  Racing first calls both look it up and store the same
// value.
static void* select_static_scratch() {
  static std::atomic<void*> ptr[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) return nullptr;
  void* p = dev < 64 ? ptr[dev].load(std::memory_order_acquire) : nullptr;
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    if (dev < 64) ptr[dev].store(p, std::memory_order_release);
  }
  return p;
}

int launch_select_static(const float* scores, int d_ff, int k, int32_t* idx, int32_t* perm, int32_t* nan_flag,
                         hipStream_t st) {
  void* ws = select_static_scratch();
  if (!ws) return -1;
  // nothing in the scratch has to start at zero: every key, candidate key and candidate index
  // that a launch reads was written earlier in the same call
  return launch_select(scores, d_ff, k, idx, perm, nan_flag, ws, st);
}

}  // namespace ffsplit
