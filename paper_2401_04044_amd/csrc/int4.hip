// Group-wise int4 remainder (round-to-nearest, group 128 along d_model; Sec. 5.2)
// with a dense bf16 heavy part: build-time packing and the weight-streaming
// decode kernels for up to 16 tokens per pass.
//
// The decode is HBM-bound: every weight byte is read once, with 16-byte loads
// that are contiguous across the wavefront, dequantised in registers and fed to
// v_mfma_f32_16x16x32_bf16 with the (at most 16) tokens as the other operand.
//
// Blocks.  One 1 KiB block holds 16 rows x 128 reduction elements of int4
// codes: lane l = 16 q + r (r = row, q = 0..3) owns 16 bytes = 4 dwords; dword s
// covers the reduction elements 32 s + 8 q + e (e = 0..7), stored offset-binary
// (code + 8) with element e = 2 i in nibble i and e = 2 i + 1 in nibble 4 + i, so
// that (dword >> 4 i) & 0x000F000F | 0x43004300 is the bf16 pair (128 + c_2i,
// 128 + c_2i+1): one MFMA operand register per and-or.  The constant 136 = 128 + 8
// is removed after the product (sum of activations times 136).
//   up/gate : rows = 16 neurons, reduction = 128 inputs of one quantisation group;
//             blocks ordered [neuron tile][group]; scales [tile][group][16] fp16.
//   down    : rows = 16 outputs c, reduction = 128 neurons; blocks ordered
//             [c group of 128][neuron block][c tile of 16]; scales [c group][neuron]
//             fp16 (the down row of a neuron is quantised in groups along c, so its
//             scale multiplies the neuron's activation before the product).
// Heavy bf16 weights use the same block order with 4 KiB blocks (one 16-byte
// MFMA operand per lane and 32-element step).
#include "int4.h"
#include <type_traits>

namespace ffsplit {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

union Frag {
  uint4 u;
  bf16x8_t v;
  uint32_t w[4];
};

__device__ __forceinline__ Frag dequant8(uint32_t w) {
  Frag f;
#pragma unroll
  for (int p = 0; p < 4; ++p) f.w[p] = ((w >> (4 * p)) & 0x000F000Fu) | 0x43004300u;
  return f;
}

__device__ __forceinline__ float half_bits_to_f32(uint16_t h) {
  _Float16 x;
  __builtin_memcpy(&x, &h, 2);
  return (float)x;
}

// round-to-nearest symmetric int4 code of w for scale s (all fp32), offset-binary
__device__ __forceinline__ uint32_t quant_code(float w, float s) {
  int q = 0;
  if (s > 0.f) {
    float t = rintf(w / s);
    t = fminf(fmaxf(t, -8.f), 7.f);
    q = (int)t;
  }
  return (uint32_t)(q + 8) & 15u;
}

__device__ __forceinline__ float group_scale(float amax, uint16_t* bits) {
  const _Float16 h = (_Float16)(amax / 7.0f);
  __builtin_memcpy(bits, &h, 2);
  return (float)h;
}

// ---------------------------------------------------------------- remainder order

__global__ void __launch_bounds__(1024) rest_order_kernel(const int32_t* idx, int k, int n, int32_t* rest,
                                                          int32_t* flags) {
  __shared__ int wsum[16];
  const int tid = threadIdx.x;
  for (int i = tid; i < n; i += 1024) flags[i] = 0;
  __syncthreads();
  for (int i = tid; i < k; i += 1024) flags[idx[i]] = 1;
  __syncthreads();
  int base_out = 0;
  for (int base = 0; base < n; base += 1024) {
    const int i = base + tid;
    const bool keep = i < n && flags[i] == 0;
    int tot;
    const int pos = base_out + block_prefix_1024(keep, wsum, &tot);
    base_out += tot;
    if (keep) rest[pos] = i;
  }
}

int launch_rest_order(const int32_t* idx, int k, int d_ff, int32_t* rest, int32_t* flags, hipStream_t st) {
  hipLaunchKernelGGL(rest_order_kernel, dim3(1), dim3(1024), 0, st, idx, k, d_ff, rest, flags);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ---------------------------------------------------------------- packing

// up / gate: W [d, d_ff] bf16, neuron jj of the remainder = column rest[jj]
__global__ void __launch_bounds__(256) pack_up_int4_kernel(const bf16_t* W, int d_ff, const int32_t* rest, int m,
                                                           int G, uint32_t* nib, uint16_t* sc) {
  __shared__ float tile[128][17];
  __shared__ float pm[16][16];
  __shared__ float sf[16];
  const int nt = blockIdx.x, g = blockIdx.y, tid = threadIdx.x;
  {
    const int n = tid & 15, kk0 = tid >> 4;
    const int jj = nt * 16 + n;
    const int col = jj < m ? rest[jj] : -1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int kk = kk0 + 16 * i;
      tile[kk][n] = col >= 0 ? bf16_to_f32(W[(int64_t)(g * 128 + kk) * d_ff + col]) : 0.f;
    }
  }
  __syncthreads();
  {
    const int n = tid & 15, part = tid >> 4;
    float mx = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(tile[part * 8 + i][n]));
    pm[part][n] = mx;
  }
  __syncthreads();
  if (tid < 16) {
    float a = 0.f;
    for (int pp = 0; pp < 16; ++pp) a = fmaxf(a, pm[pp][tid]);
    uint16_t bits;
    sf[tid] = group_scale(a, &bits);
    sc[((int64_t)nt * G + g) * 16 + tid] = bits;
  }
  __syncthreads();
  const int lane = tid >> 2, s = tid & 3, r = lane & 15, q = lane >> 4;
  const float scale = sf[r];
  uint32_t dw = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t c = quant_code(tile[32 * s + 8 * q + e][r], scale);
    const int pos = (e & 1) ? 4 + (e >> 1) : (e >> 1);
    dw |= c << (4 * pos);
  }
  nib[(((int64_t)nt * G + g) * 64 + lane) * 4 + s] = dw;
}

// down: W2 [d_ff, d] bf16, neuron jj = row rest[jj]; groups run along the row
__global__ void __launch_bounds__(256) pack_down_int4_kernel(const bf16_t* W2, int d, const int32_t* rest, int m,
                                                             int JB, int jp128, uint32_t* nib, uint16_t* sc) {
  __shared__ uint16_t tile[128][136];
  __shared__ float sf[128];
  const int cg = blockIdx.x, jb = blockIdx.y, tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (tid >> 4) + 16 * i, chunk = tid & 15;
    const int jj = jb * 128 + row;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (jj < m) v = *(const uint4*)(W2 + (int64_t)rest[jj] * d + cg * 128 + chunk * 8);
    *(uint4*)&tile[row][chunk * 8] = v;
  }
  __syncthreads();
  if (tid < 128) {
    float a = 0.f;
    for (int c = 0; c < 128; ++c) a = fmaxf(a, fabsf(bf16_to_f32(tile[tid][c])));
    uint16_t bits;
    sf[tid] = group_scale(a, &bits);
    sc[(int64_t)cg * jp128 + jb * 128 + tid] = bits;
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int id = tid + 256 * it;
    const int ct = id >> 8, rem = id & 255, lane = rem >> 2, s = rem & 3, r = lane & 15, q = lane >> 4;
    uint32_t dw = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int j = 32 * s + 8 * q + e;
      const uint32_t c = quant_code(bf16_to_f32(tile[j][ct * 16 + r]), sf[j]);
      const int pos = (e & 1) ? 4 + (e >> 1) : (e >> 1);
      dw |= c << (4 * pos);
    }
    nib[((((int64_t)cg * JB + jb) * 8 + ct) * 64 + lane) * 4 + s] = dw;
  }
}

// heavy up/gate in decode order: chunk ((ht*G + g)*4 + s)*64 + lane holds the 8 inputs
// g*128 + 32 s + 8 q + e of heavy neuron ht*16 + r
__global__ void pack_heavy_up_kernel(const bf16_t* W, int d_ff, const int32_t* idx, int k, int G, int n_chunks,
                                     uint4* out) {
  const int id = blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= n_chunks) return;
  const int lane = id & 63, s = (id >> 6) & 3, tg = id >> 8;
  const int g = tg % G, ht = tg / G, r = lane & 15, q = lane >> 4;
  const int pos = ht * 16 + r;
  uint16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int kk = g * 128 + 32 * s + 8 * q + e;
    v[e] = pos < k ? W[(int64_t)kk * d_ff + idx[pos]] : (uint16_t)0;
  }
  out[id] = make_uint4(v[0] | (uint32_t)v[1] << 16, v[2] | (uint32_t)v[3] << 16, v[4] | (uint32_t)v[5] << 16,
                       v[6] | (uint32_t)v[7] << 16);
}

// heavy down in decode order: chunk ((((cg*JBh + jb)*8 + ct)*4 + s)*64 + lane) holds
// W2[idx[jb*128 + 32 s + 8 q + e]][cg*128 + ct*16 + r]
__global__ void pack_heavy_down_kernel(const bf16_t* W2, int d, const int32_t* idx, int k, int JBh, int n_chunks,
                                       uint4* out) {
  const int id = blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= n_chunks) return;
  const int lane = id & 63, s = (id >> 6) & 3, ct = (id >> 8) & 7, t = id >> 11;
  const int jb = t % JBh, cg = t / JBh, r = lane & 15, q = lane >> 4;
  const int c = cg * 128 + ct * 16 + r;
  uint16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int j = jb * 128 + 32 * s + 8 * q + e;
    v[e] = j < k ? W2[(int64_t)idx[j] * d + c] : (uint16_t)0;
  }
  out[id] = make_uint4(v[0] | (uint32_t)v[1] << 16, v[2] | (uint32_t)v[3] << 16, v[4] | (uint32_t)v[5] << 16,
                       v[6] | (uint32_t)v[7] << 16);
}

int launch_int4_pack(const ffsplit_desc_t& d, const Layout& L, const void* W1, const void* Wg, const void* W2,
                     const int32_t* rest, const int32_t* idx, char* split, hipStream_t st) {
  const int m = d.d_ff - d.k, G = L.groups, dm = d.d_model;
  const void* ups[2] = {W1, Wg};
  for (int w = 0; w < L.n_up; ++w) {
    if (m > 0) {
      hipLaunchKernelGGL(pack_up_int4_kernel, dim3(L.jp16 / 16, G), dim3(256), 0, st, (const bf16_t*)ups[w], d.d_ff,
                         rest, m, G, (uint32_t*)(split + L.off_i4[w]), (uint16_t*)(split + L.off_s4[w]));
      if (hipGetLastError() != hipSuccess) return -1;
    }
    if (d.k > 0) {
      const int n_chunks = (L.kp / 16) * G * 4 * 64;
      hipLaunchKernelGGL(pack_heavy_up_kernel, dim3((n_chunks + 255) / 256), dim3(256), 0, st,
                         (const bf16_t*)ups[w], d.d_ff, idx, d.k, G, n_chunks, (uint4*)(split + L.off_hv[w]));
      if (hipGetLastError() != hipSuccess) return -1;
    }
  }
  if (m > 0) {
    const int JB = L.jp128 / 128;
    hipLaunchKernelGGL(pack_down_int4_kernel, dim3(G, JB), dim3(256), 0, st, (const bf16_t*)W2, dm, rest, m, JB,
                       L.jp128, (uint32_t*)(split + L.off_i4[2]), (uint16_t*)(split + L.off_s4[2]));
    if (hipGetLastError() != hipSuccess) return -1;
  }
  if (d.k > 0) {
    const int JBh = L.kp128 / 128;
    const int n_chunks = G * JBh * 8 * 4 * 64;
    hipLaunchKernelGGL(pack_heavy_down_kernel, dim3((n_chunks + 255) / 256), dim3(256), 0, st, (const bf16_t*)W2, dm,
                       idx, d.k, JBh, n_chunks, (uint4*)(split + L.off_hv[2]));
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

// ---------------------------------------------------------------- export (test hook)

__global__ void export_int4_kernel(const uint32_t* nib, const uint16_t* sc, int what, int m, int d, int G, int JB,
                                   int jp128, int8_t* q_out, uint16_t* s_out) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)m * d) return;
  const int jj = (int)(id / d), c = (int)(id % d);
  uint32_t dw;
  int e;
  uint16_t sbits;
  if (what != 2) {
    const int nt = jj >> 4, r = jj & 15, g = c >> 7, kk = c & 127, s = kk >> 5, q = (kk & 31) >> 3;
    e = kk & 7;
    dw = nib[(((int64_t)nt * G + g) * 64 + q * 16 + r) * 4 + s];
    sbits = sc[((int64_t)nt * G + g) * 16 + r];
    if (kk == 0) s_out[(int64_t)jj * G + g] = sbits;
  } else {
    const int cg = c >> 7, ct = (c & 127) >> 4, r = c & 15, jb = jj >> 7, jl = jj & 127, s = jl >> 5,
              q = (jl & 31) >> 3;
    e = jl & 7;
    dw = nib[((((int64_t)cg * JB + jb) * 8 + ct) * 64 + q * 16 + r) * 4 + s];
    sbits = sc[(int64_t)cg * jp128 + jj];
    if ((c & 127) == 0) s_out[(int64_t)jj * G + cg] = sbits;
  }
  const int pos = (e & 1) ? 4 + (e >> 1) : (e >> 1);
  q_out[id] = (int8_t)((int)((dw >> (4 * pos)) & 15u) - 8);
}

int launch_int4_export(const ffsplit_desc_t& d, const Layout& L, const char* split, int what, int8_t* q_out,
                       uint16_t* s_out, hipStream_t st) {
  const int m = d.d_ff - d.k;
  if (m <= 0) return 0;
  const int64_t n = (int64_t)m * d.d_model;
  hipLaunchKernelGGL(export_int4_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     (const uint32_t*)(split + L.off_i4[what]), (const uint16_t*)(split + L.off_s4[what]), what, m,
                     d.d_model, L.groups, L.jp128 / 128, L.jp128, q_out, s_out);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ---------------------------------------------------------------- decode
// Up to 16 tokens per pass, HBM-bound: every weight byte is read once with 16-byte loads
// that are contiguous across the wavefront, dequantised in registers and fed to
// v_mfma_f32_16x16x32_bf16 with the tokens as the other operand.  Both kernels request
// their weights before anything else so that one memory latency covers the whole
// workgroup's share.
//
// phase 1   h[t, j] = act(x_t . up_j [, x_t . gate_j]) for every neuron (bf16).
//           A workgroup of 8 wavefronts owns one heavy tile of 16 neurons or TPW int4
//           tiles; wavefront w owns the quantisation groups w*GPW.. of the reduction and
//           keeps the tokens' activations for them in registers; the 8 partial 16x16
//           results are added in a fixed order through LDS.
// phase 2   y[t, c] = sum_j h[t, j] * down[j, c].  Workgroup (cg, s) owns the 128 outputs
//           of column group cg and every S-th block of 128 neurons; wavefront w owns the
//           16 outputs cg*128 + 16 w.  The scaled activations (MFMA operands) of the
//           workgroup's neuron blocks are prepared once into LDS.  Partial sums are
//           written with device-scope stores; the last of the S workgroups of a column
//           group to arrive (integer arrival counter) adds them in a fixed order and
//           writes Y: no floating-point atomics, results independent of arrival order.

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

union VFrag {
  u32x4_t u;
  bf16x8_t v;
  uint32_t w[4];
};

// (a & mask) | o in one instruction: the compiler emits an and and an or, and the unpack is most
// of phase 1's vector arithmetic
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t o) {
  uint32_t r;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(o));
  return r;
}

__device__ __forceinline__ VFrag dequant8v(uint32_t w) {
  VFrag f;
#pragma unroll
  for (int p = 0; p < 4; ++p) f.w[p] = and_or(w >> (4 * p), 0x000F000Fu, 0x43004300u);
  return f;
}

// partial sums cross workgroups of one launch: device-scope accesses go to the point where
// the per-XCD L2 caches are coherent, so no cache write-back or invalidate is needed;
// two adjacent floats (8-byte aligned) per access
__device__ __forceinline__ void st_dev2(float* p, float a, float b) {
  const unsigned long long v = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
  __hip_atomic_store((unsigned long long*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_dev2(const float* p) {
  const unsigned long long v = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((unsigned)v), __uint_as_float((unsigned)(v >> 32)));
}

struct Phase1Args {
  const bf16_t* X;        // [T, d]
  int T, d, G;
  int n_up;               // 1: GeLU(up)   2: silu(gate) * up
  const u32x4_t* hv_up;   // heavy bf16 blocks [tile][group][4 steps][64 lanes]
  const u32x4_t* hv_gate;
  int n_htiles;
  const u32x4_t* q_up;    // int4 blocks [tile][group][64 lanes]
  const u32x4_t* q_gate;
  const uint16_t* s_up;   // [tile][group][16] fp16
  const uint16_t* s_gate;
  int n_qtiles, tpw;      // int4 tiles per workgroup
  bf16_t* h;              // [16, hl] bf16; heavy neurons at column 0, remainder at h_off_q
  int hl, h_off_q;
  unsigned* counters;     // the second kernel's arrival counters, cleared here
  int n_counters;
};


template <int GPW, int NWV, int NUP>
__global__ void __launch_bounds__(NWV * 64) int4_phase1_kernel(const Phase1Args p) {
  // cross-wave partial sums of a tile: [tile][wave][up / gate][16 x 16]
  __shared__ float red[1][NWV][2][256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, q = lane >> 4;
  const int wg = blockIdx.x;
  const bool heavy = wg < p.n_htiles;

  // The first workgroup also clears what the second kernel expects to be zero: the arrival
  // counters, and the columns of h that no neuron writes (padding up to whole 128-blocks).
  if (wg == 0) {
    for (int i = tid; i < p.n_counters; i += NWV * 64) p.counters[i] = 0u;
    const int pad_h = p.h_off_q - p.n_htiles * 16, pad_q = p.hl - p.h_off_q - p.n_qtiles * 16;
    for (int i = tid; i < 16 * (pad_h + pad_q); i += NWV * 64) {
      const int row = i / (pad_h + pad_q), c = i % (pad_h + pad_q);
      const int col = c < pad_h ? p.n_htiles * 16 + c : p.h_off_q + p.n_qtiles * 16 + (c - pad_h);
      p.h[(int64_t)row * p.hl + col] = 0;
    }
  }

  // ---- tokens' activations for this wavefront's quantisation groups, as MFMA operands.
  // Requested before the weights (they come from cache and return first, so the per-group sums
  // below are formed while the weights are in flight); addresses are clamped and the values
  // masked so that the loads stay unconditional.
  VFrag xr[GPW][4];
  float xsum[GPW];
#pragma unroll
  for (int i = 0; i < GPW; ++i) {
    const int g = wave * GPW + i;
    const bool valid = g < p.G && n < p.T;
    const int gc = min(g, p.G - 1), nc = min(n, p.T - 1);
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const u32x4_t v = *(const u32x4_t*)(p.X + (int64_t)nc * p.d + gc * 128 + 32 * st + 8 * q);
      xr[i][st].u = valid ? v : u32x4_t{0, 0, 0, 0};
    }
  }

  // ---- then the weights.  One register buffer, refilled piecewise: as soon as the MFMAs of a
  // quantisation group (int4) or of a 32-element step (heavy) are issued, the same registers
  // are loaded with the corresponding piece of the next tile / group, so that about a tile's
  // worth of this wavefront's weights is in flight while it computes.
  constexpr int NRB = (GPW * 2 > 8) ? GPW * 2 : 8;   // 16-byte registers
  u32x4_t R[NRB];
  u32x2_t su[GPW], sg[GPW];
  const int qt0 = (wg - p.n_htiles) * p.tpw;
  const int qt_end = min(p.n_qtiles, qt0 + p.tpw);
  // (a group past the end of the reduction reads the last group's weights: its activations
  // are zero, so it adds nothing, and the code stays free of branches, which keeps the
  // compiler's memory-counter waits exact)
  auto load_q = [&](int i, int qt) {   // group i of this wavefront, tile qt
    const int g = min(wave * GPW + i, p.G - 1);
    const int64_t blk = (int64_t)qt * p.G + g;
    R[i * 2] = p.q_up[blk * 64 + lane];
    su[i] = *(const u32x2_t*)(p.s_up + blk * 16 + 4 * q);
    if (NUP == 2) {
      R[i * 2 + 1] = p.q_gate[blk * 64 + lane];
      sg[i] = *(const u32x2_t*)(p.s_gate + blk * 16 + 4 * q);
    }
  };
  auto load_h = [&](int st, int i) {   // step st of group i of this wavefront
    const int g = min(wave * GPW + i, p.G - 1);
    const int64_t at = (((int64_t)wg * p.G + g) * 4 + st) * 64 + lane;
    R[st * 2] = p.hv_up[at];
    if (NUP == 2) R[st * 2 + 1] = p.hv_gate[at];
  };
  if (heavy) {
#pragma unroll
    for (int st = 0; st < 4; ++st) load_h(st, 0);
  } else if (qt0 < qt_end) {
#pragma unroll
    for (int i = 0; i < GPW; ++i) load_q(i, qt0);
  }

#pragma unroll
  for (int i = 0; i < GPW; ++i) {
    float s = 0.f;
#pragma unroll
    for (int st = 0; st < 4; ++st)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s += __uint_as_float(xr[i][st].w[e] << 16);
        s += __uint_as_float(xr[i][st].w[e] & 0xffff0000u);
      }
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    xsum[i] = s;
  }

  // cross-wave sum of `nt` tiles' partials, activation, store of h (bf16 pairs)
  auto finish = [&](int nt, int col0, int col_step) {
    __syncthreads();
    const int t = tid >> 7, pair = tid & 127;
    if (t < nt) {
      float u0 = 0.f, g0 = 0.f, u1 = 0.f, g1 = 0.f;
#pragma unroll
      for (int w = 0; w < NWV; ++w) {
        u0 += red[t][w][0][2 * pair]; g0 += red[t][w][1][2 * pair];
        u1 += red[t][w][0][2 * pair + 1]; g1 += red[t][w][1][2 * pair + 1];
      }
      const int l = pair >> 1, r = (pair & 1) * 2;
      const int tok = l & 15, neuron = 4 * (l >> 4) + r;
      const float h0 = NUP == 2 ? silu_f(g0) * u0 : gelu_f(u0);
      const float h1 = NUP == 2 ? silu_f(g1) * u1 : gelu_f(u1);
      if (tok < p.T)
        *(uint32_t*)(p.h + (int64_t)tok * p.hl + col0 + t * col_step + neuron) = pack_bf16x2(h0, h1);
    }
  };

  if (heavy) {
    f32x4_t au = {0.f, 0.f, 0.f, 0.f}, ag = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < GPW; ++i) {
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        VFrag a, c;
        a.u = R[st * 2];
        au = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, xr[i][st].v, au, 0, 0, 0);
        if (NUP == 2) {
          c.u = R[st * 2 + 1];
          ag = __builtin_amdgcn_mfma_f32_16x16x32_bf16(c.v, xr[i][st].v, ag, 0, 0, 0);
        }
        if (i + 1 < GPW) load_h(st, i + 1);
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      red[0][wave][0][lane * 4 + r] = au[r];
      red[0][wave][1][lane * 4 + r] = ag[r];
    }
    finish(1, wg * 16, 0);
    return;
  }

  // one tile: products group by group; with REFILL the group's registers are reloaded with the
  // same group of tile qt + 1 as soon as its MFMAs are issued
  auto tile = [&](int qt, auto refill) {
    constexpr bool REFILL = decltype(refill)::value;
    f32x4_t au = {0.f, 0.f, 0.f, 0.f}, ag = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < GPW; ++i) {
      const float corr = 136.f * xsum[i];
      f32x4_t ru = {0.f, 0.f, 0.f, 0.f}, rg = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < 4; ++st)
        ru = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dequant8v(R[i * 2][st]).v, xr[i][st].v, ru, 0, 0, 0);
      if (NUP == 2) {
#pragma unroll
        for (int st = 0; st < 4; ++st)
          rg = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dequant8v(R[i * 2 + 1][st]).v, xr[i][st].v, rg, 0, 0, 0);
      }
      float fu[4], fg[4];
      fu[0] = half_bits_to_f32((uint16_t)(su[i][0] & 0xffffu)); fu[1] = half_bits_to_f32((uint16_t)(su[i][0] >> 16));
      fu[2] = half_bits_to_f32((uint16_t)(su[i][1] & 0xffffu)); fu[3] = half_bits_to_f32((uint16_t)(su[i][1] >> 16));
      if (NUP == 2) {
        fg[0] = half_bits_to_f32((uint16_t)(sg[i][0] & 0xffffu)); fg[1] = half_bits_to_f32((uint16_t)(sg[i][0] >> 16));
        fg[2] = half_bits_to_f32((uint16_t)(sg[i][1] & 0xffffu)); fg[3] = half_bits_to_f32((uint16_t)(sg[i][1] >> 16));
      }
      if (REFILL) load_q(i, qt + 1);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        au[r] = fmaf(fu[r], ru[r] - corr, au[r]);
        if (NUP == 2) ag[r] = fmaf(fg[r], rg[r] - corr, ag[r]);
      }
      __builtin_amdgcn_sched_barrier(0);   // one group at a time: keeps the dequantised operands few
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      red[0][wave][0][lane * 4 + r] = au[r];
      red[0][wave][1][lane * 4 + r] = ag[r];
    }
  };
  int qt = qt0;
  for (; qt + 1 < qt_end; ++qt) {
    tile(qt, std::true_type{});
    finish(1, p.h_off_q + qt * 16, 16);
    __syncthreads();   // red is reused
  }
  if (qt < qt_end) {
    tile(qt, std::false_type{});
    finish(1, p.h_off_q + qt * 16, 16);
  }
}

// 16-byte global load whose completion the kernel tracks itself: the compiler neither waits for
// it nor moves it; every use is preceded by wait_loads<N>(reg), which waits until at most the N
// most recently issued vector-memory operations are outstanding and ties the register to the wait.
__device__ __forceinline__ u32x4_t load16_untracked(const void* ptr) {
  u32x4_t v;
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(ptr) : "memory");
  return v;
}
template <int N>
__device__ __forceinline__ void wait_loads(u32x4_t& r) {
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(r) : "n"(N) : "memory");
}

template <int I, int END, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < END) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, END>(f);
  }
}

struct Phase2Args {
  const bf16_t* h;         // [16, hl]
  int T, d, hl, h_off_q, S;
  const u32x4_t* hv_down;  // [cg][JBh][8 ct][4 steps][64]
  int JBh;
  const u32x4_t* q_down;   // [cg][JBr][8 ct][64]
  const uint16_t* s_down;  // [cg][jp128] fp16
  int JBr, jp128;
  float* part;             // [G][S][2][16][128] fp32 (heavy, remainder)
  unsigned* counters;      // [G] arrivals, zero on entry
  bf16_t* Y;
  bf16_t* Yh;
  bf16_t* Yr;
  const float* b2;         // [d] output bias or null
  const float* resid;      // [T, d] residual stream or null
  int out_f32;             // Y holds fp32
};

constexpr int P2_MAXJ = 12;  // int4 neuron blocks per workgroup and pass
constexpr int P2_MAXH = 4;   // heavy 32-neuron steps per workgroup and pass
constexpr int P2_STEPS = P2_MAXJ * 4 + P2_MAXH;

__global__ void __launch_bounds__(512) int4_phase2_kernel(const Phase2Args p) {
  __shared__ u32x4_t hop[P2_STEPS][64];
  __shared__ float hsum_s[8][16];
  __shared__ int flag_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, q = lane >> 4;
  const int cg = blockIdx.x, sp = blockIdx.y;

  const int NJ = p.JBr > sp ? (p.JBr - sp + p.S - 1) / p.S : 0;           // int4 blocks sp, sp+S, ...
  const int NHq = p.JBh * 4 > sp ? (p.JBh * 4 - sp + p.S - 1) / p.S : 0;  // heavy steps sp, sp+S, ...
  // Loads are kept free of branches (indices past the end are clamped to the last valid block:
  // a repeated address, served by the cache) so that the compiler's memory-counter waits stay
  // exact and the small activation loads below need not wait for the weights behind them.
  u32x4_t w2[P2_MAXJ], wh[P2_MAXH];
  // (a part with no block at all for this workgroup reads the start of the other part's
  // blocks instead, which exist: d_ff > 0)
  const u32x4_t* qsrc = NJ > 0 ? p.q_down : p.hv_down;
  const u32x4_t* hsrc = NHq > 0 ? p.hv_down : p.q_down;
  auto load_down = [&](int pass) {
#pragma unroll
    for (int i = 0; i < P2_MAXJ; ++i) {
      const int ii = min(pass * P2_MAXJ + i, NJ - 1);
      const int64_t at = NJ > 0 ? (((int64_t)cg * p.JBr + sp + ii * p.S) * 8 + wave) * 64 + lane : tid;
      w2[i] = load16_untracked(qsrc + at);
    }
#pragma unroll
    for (int i = 0; i < P2_MAXH; ++i) {
      const int hq = sp + min(pass * P2_MAXH + i, NHq - 1) * p.S;
      const int64_t at = NHq > 0 ? ((((int64_t)cg * p.JBh + (hq >> 2)) * 8 + wave) * 4 + (hq & 3)) * 64 + lane : tid;
      wh[i] = load16_untracked(hsrc + at);
    }
  };

  f32x4_t acc_r = {0.f, 0.f, 0.f, 0.f}, acc_h = {0.f, 0.f, 0.f, 0.f};
  float hsum = 0.f;
  const int n_pass_j = (NJ + P2_MAXJ - 1) / P2_MAXJ, n_pass_h = (NHq + P2_MAXH - 1) / P2_MAXH;
  const int n_pass = n_pass_j > n_pass_h ? n_pass_j : n_pass_h;
  constexpr int HPW = (P2_STEPS + 7) / 8;   // operand steps prepared per wavefront and pass
  for (int pass = 0; pass < n_pass; ++pass) {
    if (pass > 0) __syncthreads();   // hop is reused
    const int nj = max(0, min(P2_MAXJ, NJ - pass * P2_MAXJ));
    const int nh = max(0, min(P2_MAXH, NHq - pass * P2_MAXH));
    const int n_steps = nj * 4 + nh;
    // 1. the activations (and, for the int4 part, the neurons' scales for this column group) of
    //    this wavefront's operand steps: step sigma < 4 nj is (int4 block sigma / 4, 32-neuron
    //    step sigma % 4), the rest heavy.  Requested before the weights: they come from cache
    //    and return first.
    u32x4_t hreg[HPW], sreg[HPW];
#pragma unroll
    for (int i = 0; i < HPW; ++i) {
      const int sgm = min(wave + 8 * i, n_steps - 1);
      const bool hv = sgm >= nj * 4;
      const int jq = sp + (pass * P2_MAXJ + (sgm >> 2)) * p.S;
      const int hq = sp + (pass * P2_MAXH + (sgm - nj * 4)) * p.S;
      const int j0 = hv ? (hq >> 2) * 128 + 32 * (hq & 3) + 8 * q : jq * 128 + 32 * (sgm & 3) + 8 * q;
      const int tok = n < p.T ? n : 0;
      hreg[i] = load16_untracked(p.h + (int64_t)tok * p.hl + (hv ? 0 : p.h_off_q) + j0);
      sreg[i] = load16_untracked(p.s_down + (int64_t)cg * p.jp128 + (hv ? 0 : j0));
    }
    // 2. the weights
    load_down(pass);
    // 3. operands into LDS (the P2_MAXJ + P2_MAXH weight loads may still be in flight)
#pragma unroll
    for (int i = 0; i < HPW; ++i) {
      wait_loads<P2_MAXJ + P2_MAXH>(hreg[i]);
      wait_loads<P2_MAXJ + P2_MAXH>(sreg[i]);
    }
#pragma unroll
    for (int i = 0; i < HPW; ++i) {
      const int sgm = wave + 8 * i;
      const bool hv = sgm >= nj * 4;
      VFrag f;
      f.u = hreg[i];
      float part = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // the down row of a neuron is quantised in groups along the outputs: its scale for this
        // column group multiplies the neuron's activation
        const float lo = __uint_as_float(f.w[e] << 16) * half_bits_to_f32((uint16_t)(sreg[i][e] & 0xffffu));
        const float hi = __uint_as_float(f.w[e] & 0xffff0000u) * half_bits_to_f32((uint16_t)(sreg[i][e] >> 16));
        const uint32_t sc = pack_bf16x2(lo, hi);
        part += __uint_as_float(sc << 16) + __uint_as_float(sc & 0xffff0000u);
        f.w[e] = hv ? f.w[e] : sc;
      }
      if (n >= p.T) { f.u = u32x4_t{0, 0, 0, 0}; part = 0.f; }
      if (sgm < n_steps) {
        hop[sgm][lane] = f.u;
        if (!hv) hsum += part;
      }
    }
    __syncthreads();
    static_for<0, P2_MAXJ>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      wait_loads<P2_MAXJ - 1 - i + P2_MAXH>(w2[i]);
      if (i < nj) {
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          VFrag b;
          b.u = hop[i * 4 + st][lane];
          acc_r = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dequant8v(w2[i][st]).v, b.v, acc_r, 0, 0, 0);
        }
      }
    });
    static_for<0, P2_MAXH>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      wait_loads<P2_MAXH - 1 - i>(wh[i]);
      if (i < nh) {
        VFrag a, b;
        a.u = wh[i];
        b.u = hop[nj * 4 + i][lane];
        acc_h = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, acc_h, 0, 0, 0);
      }
    });
  }
  // the constant 136 of the offset-binary codes: subtract 136 * (sum of this workgroup's scaled activations)
  hsum += __shfl_xor(hsum, 16);
  hsum += __shfl_xor(hsum, 32);
  if (q == 0) hsum_s[wave][n] = hsum;
  __syncthreads();
  {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 8; ++w) tot += hsum_s[w][n];
    const float corr = 136.f * tot;
#pragma unroll
    for (int r = 0; r < 4; ++r) acc_r[r] -= corr;
  }
  // lane holds outputs c = 16 wave + 4 q + r of token n.  Unless the caller wants the heavy
  // and the remainder parts separately, only their sum crosses workgroups.
  const bool parts = p.Yh != nullptr || p.Yr != nullptr;
  float* pw = p.part + ((int64_t)(cg * p.S + sp) * 2) * 16 * 128 + n * 128 + wave * 16 + 4 * q;
  if (parts) {
    st_dev2(pw, acc_h[0], acc_h[1]);
    st_dev2(pw + 2, acc_h[2], acc_h[3]);
    st_dev2(pw + 16 * 128, acc_r[0], acc_r[1]);
    st_dev2(pw + 16 * 128 + 2, acc_r[2], acc_r[3]);
  } else {
    st_dev2(pw, acc_h[0] + acc_r[0], acc_h[1] + acc_r[1]);
    st_dev2(pw + 2, acc_h[2] + acc_r[2], acc_h[3] + acc_r[3]);
  }
  // Hand-off to the last arriver.  The partials were written with device-scope (sc1,
  // write-through) stores, which count as complete only once they have reached the level where
  // all XCDs see them: every thread waits for its own stores (vmcnt 0) before the barrier, and
  // only after the barrier does thread 0 count this workgroup in.  The workgroup that reads
  // S - 1 then loads the partials with device-scope loads, issued after the barrier that
  // publishes the flag.  (Agent-scope release / acquire fences are correct too, but they write
  // back and invalidate the whole L2 per workgroup: 24 -> 42 us for the step.)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0)
    flag_s = __hip_atomic_fetch_add(&p.counters[cg], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(p.S - 1);
  __syncthreads();
  if (!flag_s) return;
  // last workgroup of the column group: fixed-order sum over the splits, two outputs per thread
  for (int o = 2 * tid; o < 16 * 128; o += 1024) {
    const int tok = o >> 7, c = o & 127;
    if (tok >= p.T) continue;
    // all loads first (independent), then the sums
    float2 va[16], vb[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      va[s] = make_float2(0.f, 0.f); vb[s] = make_float2(0.f, 0.f);
      if (s < p.S) {
        const float* ps = p.part + ((int64_t)(cg * p.S + s) * 2) * 16 * 128;
        va[s] = ld_dev2(ps + o);
        if (parts) vb[s] = ld_dev2(ps + 16 * 128 + o);
      }
    }
    float a0 = 0.f, a1 = 0.f, b0 = 0.f, b1 = 0.f;
#pragma unroll
    for (int s = 0; s < 16; ++s) { a0 += va[s].x; a1 += va[s].y; b0 += vb[s].x; b1 += vb[s].y; }
    const int64_t oi = (int64_t)tok * p.d + cg * 128 + c;
    float y0 = a0 + b0, y1 = a1 + b1;
    if (p.b2) { y0 += p.b2[cg * 128 + c]; y1 += p.b2[cg * 128 + c + 1]; }
    if (p.resid) { y0 += p.resid[oi]; y1 += p.resid[oi + 1]; }
    if (p.out_f32) *(float2*)((float*)p.Y + oi) = make_float2(y0, y1);
    else *(uint32_t*)(p.Y + oi) = pack_bf16x2(y0, y1);
    if (p.Yh) *(uint32_t*)(p.Yh + oi) = pack_bf16x2(a0, a1);
    if (p.Yr) *(uint32_t*)(p.Yr + oi) = pack_bf16x2(b0, b1);
  }
}

// ---------------------------------------------------------------- expansion for large batches

struct ExpandArgs {
  const u32x4_t* hv[3];      // heavy bf16 blocks: up, gate, down
  const uint32_t* nib[3];    // int4 codes
  const uint16_t* sc[3];     // fp16 group scales
  int n_up, G, d;
  int kp16, kp128, jp16, jp128;   // padded counts of the int4 layout
  int kpD, mpD, k4D;              // padded counts of the DENSE layout
  int64_t n_chunks;
  u32x4_t* out;
};

// eight codes of one dword (element e = 2 i in nibble i, e = 2 i + 1 in nibble 4 + i) times
// their scales -> eight bf16
__device__ __forceinline__ u32x4_t expand8(uint32_t dw, const float* s) {
  u32x4_t o;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = (float)((int)((dw >> (4 * i)) & 15u) - 8) * s[2 * i];
    const float hi = (float)((int)((dw >> (4 * (4 + i))) & 15u) - 8) * s[2 * i + 1];
    o[i] = pack_bf16x2(lo, hi);
  }
  return o;
}

// B1t image [n_up (kpD + mpD), d], tiled: one thread per 16-byte chunk (row, 8 inputs)
__global__ void __launch_bounds__(256) expand_up_kernel(const ExpandArgs a) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= a.n_chunks) return;
  const int lane = (int)(id & 63);
  const int64_t blk = id >> 6;
  const int kbs = a.d / 16;
  const int rb = (int)(blk / kbs), kb = (int)(blk % kbs);
  const int row = rb * 32 + (lane & 31), k0 = kb * 16 + 8 * (lane >> 5);
  const int heavy_rows = a.n_up * a.kpD;
  const bool heavy = row < heavy_rows;
  const int rr = heavy ? row : row - heavy_rows;
  // SwiGLU: 32-row blocks alternate gate / up
  const int which = a.n_up == 2 ? (((rr >> 5) & 1) ? 0 : 1) : 0;   // index into hv / nib / sc: 0 up, 1 gate
  const int n = a.n_up == 2 ? ((rr >> 6) * 32 + (rr & 31)) : rr;
  const int g = k0 >> 7, s = (k0 & 127) >> 5, q = (k0 & 31) >> 3, r16 = n & 15, t16 = n >> 4;
  u32x4_t o = {0, 0, 0, 0};
  if (heavy) {
    if (n < a.kp16) o = a.hv[which][(((int64_t)t16 * a.G + g) * 4 + s) * 64 + q * 16 + r16];
  } else if (n < a.jp16) {
    const uint32_t dw = a.nib[which][(((int64_t)t16 * a.G + g) * 64 + q * 16 + r16) * 4 + s];
    const float sc = half_bits_to_f32(a.sc[which][((int64_t)t16 * a.G + g) * 16 + r16]);
    const float ss[8] = {sc, sc, sc, sc, sc, sc, sc, sc};
    o = expand8(dw, ss);
  }
  a.out[id] = o;
}

// B4t image [d, kpD + mpD], tiled: one thread per 16-byte chunk (output c, 8 neurons)
__global__ void __launch_bounds__(256) expand_down_kernel(const ExpandArgs a) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= a.n_chunks) return;
  const int lane = (int)(id & 63);
  const int64_t blk = id >> 6;
  const int kbs = a.k4D / 16;
  const int rb = (int)(blk / kbs), kb = (int)(blk % kbs);
  const int c = rb * 32 + (lane & 31), col0 = kb * 16 + 8 * (lane >> 5);
  const int cg = c >> 7, ct = (c & 127) >> 4, r16 = c & 15;
  u32x4_t o = {0, 0, 0, 0};
  if (c < a.d) {
    if (col0 < a.kpD) {
      const int j0 = col0;
      if (j0 < a.kp128) {
        const int jb = j0 >> 7, s = (j0 & 127) >> 5, q = (j0 & 31) >> 3;
        o = a.hv[2][(((((int64_t)cg * (a.kp128 / 128) + jb) * 8 + ct) * 4 + s) * 64) + q * 16 + r16];
      }
    } else {
      const int j0 = col0 - a.kpD;
      if (j0 < a.jp128) {
        const int jb = j0 >> 7, s = (j0 & 127) >> 5, q = (j0 & 31) >> 3;
        const uint32_t dw = a.nib[2][((((int64_t)cg * (a.jp128 / 128) + jb) * 8 + ct) * 64 + q * 16 + r16) * 4 + s];
        const uint4 sb = *(const uint4*)(a.sc[2] + (int64_t)cg * a.jp128 + j0);
        const uint32_t sw[4] = {sb.x, sb.y, sb.z, sb.w};
        float ss[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          ss[2 * i] = half_bits_to_f32((uint16_t)(sw[i] & 0xffffu));
          ss[2 * i + 1] = half_bits_to_f32((uint16_t)(sw[i] >> 16));
        }
        o = expand8(dw, ss);
      }
    }
  }
  a.out[id] = o;
}

int launch_int4_expand(const ffsplit_desc_t& d, const Layout& L, const Layout& LD, const char* split, char* image,
                       hipStream_t st) {
  if (!LD.tiled || LD.dk != d.d_model || LD.dn != d.d_model) return -1;   // d_model is a multiple of 128 here
  ExpandArgs a = {};
  for (int w = 0; w < 3; ++w) {
    a.hv[w] = (const u32x4_t*)(split + L.off_hv[w]);
    a.nib[w] = (const uint32_t*)(split + L.off_i4[w]);
    a.sc[w] = (const uint16_t*)(split + L.off_s4[w]);
  }
  a.n_up = L.n_up; a.G = L.groups; a.d = d.d_model;
  a.kp16 = d.k > 0 ? L.kp : 0; a.kp128 = d.k > 0 ? L.kp128 : 0;
  a.jp16 = d.d_ff > d.k ? L.jp16 : 0; a.jp128 = d.d_ff > d.k ? L.jp128 : 0;
  a.kpD = LD.kp; a.mpD = LD.mp; a.k4D = LD.k4;
  if (LD.n1 > 0) {
    a.n_chunks = (int64_t)LD.n1 * d.d_model / 8;
    a.out = (u32x4_t*)(image + LD.off_b1);
    hipLaunchKernelGGL(expand_up_kernel, dim3((unsigned)((a.n_chunks + 255) / 256)), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  if (LD.k4 > 0) {
    a.n_chunks = (int64_t)LD.dn * LD.k4 / 8;
    a.out = (u32x4_t*)(image + LD.off_b4);
    hipLaunchKernelGGL(expand_down_kernel, dim3((unsigned)((a.n_chunks + 255) / 256)), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

static int phase2_splits(int G) {
  int S = 256 / (G > 0 ? G : 1);   // about one 8-wave workgroup per CU
  if (S > 16) S = 16;
  if (S < 1) S = 1;
  return S;
}

FwdWs make_fwd_ws(const ffsplit_desc_t& d, const Layout& L, int64_t T) {
  FwdWs w = {};
  if (d.rem_kind == FFSPLIT_REM_W3H8 && T <= W3H8_DECODE_MAX_T) {
    size_t off = 0;
    w.t_pad = 32;
    w.off_cat = off; off = align256(off + (size_t)32 * (L.k4 > 0 ? L.k4 : 16) * 2);
    int n_max = L.n_up * L.k4;
    if (L.dn > n_max) n_max = L.dn;
    w.off_kpart = off; off = align256(off + skinny_q_part_bytes(n_max));
    w.total_bytes = off;
    return w;
  }
  if ((d.rem_kind == FFSPLIT_REM_INT4 && T > INT4_DECODE_MAX_T) || d.rem_kind == FFSPLIT_REM_W3H8) {
    ffsplit_desc_t dd = d;
    dd.rem_kind = FFSPLIT_REM_DENSE;
    const Layout LD = make_layout(dd);
    w.i4_prefill = 1;
    w.off_img = 0;
    w.off_dense = align256(LD.total_bytes);
    w.total_bytes = w.off_dense + make_fwd_ws(dd, LD, T).total_bytes;
    return w;
  }
  if (d.rem_kind == FFSPLIT_REM_INT4) {
    const int hl = L.kp128 + L.jp128;
    const int S = phase2_splits(L.groups);
    size_t off = 0;
    // h and the arrival counters are adjacent: one fill zeroes both
    w.off_h = off; off = align256(off + (size_t)16 * (hl > 0 ? hl : 1) * 2);
    w.off_cnt = off; off = align256(off + (size_t)L.groups * 4);
    w.off_part = off; off = align256(off + (size_t)L.groups * S * 2 * 16 * 128 * 4);
    w.n_split = S;
    w.total_bytes = off;
    return w;
  }
  size_t off = 0;
  w.t_pad = L.tiled ? round_up((int)T, 32) : (int)T;
  w.off_cat = off; off = align256(off + (size_t)w.t_pad * L.k4 * L.esz);
  w.off_t = off; off = align256(off + (size_t)w.t_pad * L.n_up * L.rp * L.esz);
  w.off_h2 = off; off = align256(off + (size_t)w.t_pad * L.mp * L.esz);
  w.g3_split = 1;
  w.off_kpart = off;
  if (!L.tiled && L.rp > 0 && L.mp > 0 && T > 0) {
    // fp32: the product h2 * P2 has few 64 x 64 tiles and a long reduction: split it so that
    // about 256 workgroups exist, at least 8 slabs of 16 each
    const int tiles64 = (int)((T + 63) / 64) * ((L.rp + 63) / 64);
    int sp = 256 / (tiles64 > 0 ? tiles64 : 1);
    if (sp > L.mp / 128) sp = L.mp / 128;
    if (sp > 32) sp = 32;
    if (sp < 1) sp = 1;
    w.g3_split = sp;
    size_t scratch = sp > 1 ? (size_t)sp * T * L.rp * 4 : 0;
    // the other products' own splits (f32_split)
    const int ns[3] = {L.n1, L.n_up * L.mp, L.dn};
    const int ks[3] = {L.dk, L.rp, L.k4};
    for (int i = 0; i < 3; ++i) {
      const int s2 = f32_split(T, ns[i], ks[i]);
      const size_t b = (size_t)s2 * T * ns[i] * 4;
      if (s2 > 1 && b > scratch) scratch = b;
    }
    w.kpart_bytes = scratch;
    if (scratch > 0) off = align256(off + scratch);
  } else if (!L.tiled && T > 0) {
    size_t scratch = 0;
    const int ns[2] = {L.n1, L.dn};
    const int ks[2] = {L.dk, L.k4};
    for (int i = 0; i < 2; ++i) {
      const int s2 = f32_split(T, ns[i], ks[i]);
      const size_t b = (size_t)s2 * T * ns[i] * 4;
      if (s2 > 1 && b > scratch) scratch = b;
    }
    w.kpart_bytes = scratch;
    if (scratch > 0) off = align256(off + scratch);
  }
  if (L.tiled && L.rp > 0 && L.mp > 0 && T > 0) {
    // Split the long reduction of h2 * P2 across workgroups (more splits cost more partial-sum
    // traffic than they gain: measured).  Narrow products (rank <= 512 at 4096 rows) use 128x128
    // tiles with the in-workgroup K split, one workgroup per CU; wider ones use 256x128 tiles,
    // two workgroups per CU, with the number of splits that fills the 512 slots best.
    const int tiles128 = (int)((T + 127) / 128) * ((L.rp + 127) / 128);
    const int max_sp = L.mp / 512 > 0 ? L.mp / 512 : 1;   // keep >= 8 slabs of 64 per split
    int sp;
    if (tiles128 <= 128 || T <= 1024) {
      w.g3_wide = 0;
      sp = 256 / (tiles128 > 0 ? tiles128 : 1);
    } else {
      w.g3_wide = 1;
      const int tiles256 = (int)((T + 255) / 256) * ((L.rp + 127) / 128);
      sp = 1;
      double best = 0.0;
      for (int c = 1; c <= 8; ++c) {
        const int wgs = tiles256 * c;
        const double fill = (double)wgs / (512.0 * ((wgs + 511) / 512));
        if (fill > best + 0.03) { best = fill; sp = c; }
      }
      // 256 x 320 tiles (eight wavefronts with wave tiles of 64 x 160: fewer fragment reads and
      // barriers per product than 256 x 128 on four) where the rank is a multiple of 320 and some
      // split count fills whole rounds of one workgroup per CU (C5: rank 1280, 16 x 4 tiles x 4
      // splits = 256 workgroups; 201 -> 175 us); likewise 256 x 256 tiles on eight wavefronts where
      // the rank is a multiple of 256 (the Llama shape: rank 1024, 16 x 4 x 4; 94 -> 83 us)
      if (L.rp % 320 == 0) {
        const int t320 = (int)((T + 255) / 256) * (L.rp / 320);
        for (int c = 1; c <= 8 && c <= max_sp; ++c) {
          const int wgs = t320 * c;
          if (100 * wgs / (256 * ((wgs + 255) / 256)) >= 95) { w.g3_wide = 2; sp = c; break; }
        }
      } else if (L.rp % 256 == 0) {
        const int t256 = (int)((T + 255) / 256) * (L.rp / 256);
        for (int c = 1; c <= 8 && c <= max_sp; ++c) {
          const int wgs = t256 * c;
          if (100 * wgs / (256 * ((wgs + 255) / 256)) >= 95) { w.g3_wide = 3; sp = c; break; }
        }
      }
    }
    if (sp > max_sp) sp = max_sp;
    if (sp > 16) sp = 16;
    if (sp < 1) sp = 1;
    w.g3_split = sp;
    size_t scratch = sp > 1 ? (size_t)sp * T * L.rp * 4 : 0;
    if (ffn2_fused_applies(L, T)) {
      const size_t fb = (size_t)ffn2_fused_splits((int)T, L.mp) * T * L.rp * 4;
      if (fb > scratch) scratch = fb;
    }
    if (T <= SKINNY_MAX_M) {
      // small batches take the weight-streaming kernels: room for their partial tiles
      int n_max = L.n1 > L.n_up * L.mp ? L.n1 : L.n_up * L.mp;
      if (L.dn > n_max) n_max = L.dn;
      if (L.rp > n_max) n_max = L.rp;
      const size_t sk = skinny_part_bytes(n_max, (int)T);
      if (sk > scratch) scratch = sk;
    }
    if (T > SKINNY_MAX_M && T <= 1024) {
      // a few hundred rows: products with few tiles keep split-K partials of their whole output
      // (all four products: h2 * P2 too, when its own split above came out as 1)
      const int ns[4] = {L.n1, L.n_up * L.mp, L.rp, L.dn};
      const int ks[4] = {L.dk, L.rp, L.mp, L.k4};
      for (int i = 0; i < 4; ++i) {
        const size_t b = (size_t)mid_split(T, ns[i], ks[i]) * T * round_up(ns[i], 32) * 4;
        if (mid_split(T, ns[i], ks[i]) > 1 && b > scratch) scratch = b;
      }
    }
    w.kpart_bytes = scratch;
    if (scratch > 0) off = align256(off + scratch);
  } else if (L.tiled && T > 0 && T <= SKINNY_MAX_M) {
    int n_max = L.n1 > L.dn ? L.n1 : L.dn;
    off = align256(off + skinny_part_bytes(n_max, (int)T));
  } else if (L.tiled && T > SKINNY_MAX_M && T <= 1024) {
    const int ns[2] = {L.n1, L.dn};
    const int ks[2] = {L.dk, L.k4};
    size_t scratch = 0;
    for (int i = 0; i < 2; ++i) {
      const size_t b = (size_t)mid_split(T, ns[i], ks[i]) * T * round_up(ns[i], 32) * 4;
      if (mid_split(T, ns[i], ks[i]) > 1 && b > scratch) scratch = b;
    }
    w.kpart_bytes = scratch;
    if (scratch > 0) off = align256(off + scratch);
  }
  w.total_bytes = off > 0 ? off : 256;
  return w;
}

template <int GPW, int NWV>
static int launch_phase1(const Phase1Args& a, int grid, hipStream_t st) {
  if (a.n_up == 2) hipLaunchKernelGGL((int4_phase1_kernel<GPW, NWV, 2>), dim3(grid), dim3(NWV * 64), 0, st, a);
  else hipLaunchKernelGGL((int4_phase1_kernel<GPW, NWV, 1>), dim3(grid), dim3(NWV * 64), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int int4_forward(const ffsplit_desc_t& d, const Layout& L, const FwdWs& w, const char* split, const void* X, int M,
                 void* Y, void* Y_heavy, void* Y_rem, const Epilogue& ep, char* ws, hipStream_t st) {
  const int m = d.d_ff - d.k, dm = d.d_model, G = L.groups;
  const int hl = L.kp128 + L.jp128;
  const int S = w.n_split;
  const int nwv = 8;
  const int gpw = (G + nwv - 1) / nwv;
  if (gpw > 4) return -2;
  const int n_h = L.kp / 16, n_q = m > 0 ? L.jp16 / 16 : 0;
  // int4 tiles per workgroup: about one 8-wave workgroup per CU in total, so that the tokens'
  // activations are fetched once per CU rather than once per tile
  const int slots = 256 - n_h > 32 ? 256 - n_h : 32;
  int tpw = n_q > 0 ? (n_q + slots - 1) / slots : 1;
  if (tpw < 1) tpw = 1;
  const int grid1 = n_h + (n_q + tpw - 1) / tpw;
  for (int t0 = 0; t0 < M; t0 += 16) {
    const int T = M - t0 < 16 ? M - t0 : 16;
    Phase1Args a = {};
    a.X = (const bf16_t*)X + (int64_t)t0 * dm;
    a.T = T; a.d = dm; a.G = G; a.n_up = L.n_up;
    a.hv_up = (const u32x4_t*)(split + L.off_hv[0]);
    a.hv_gate = (const u32x4_t*)(split + L.off_hv[1]);
    a.n_htiles = n_h;
    a.q_up = (const u32x4_t*)(split + L.off_i4[0]);
    a.q_gate = (const u32x4_t*)(split + L.off_i4[1]);
    a.s_up = (const uint16_t*)(split + L.off_s4[0]);
    a.s_gate = (const uint16_t*)(split + L.off_s4[1]);
    a.n_qtiles = n_q; a.tpw = tpw;
    a.h = (bf16_t*)(ws + w.off_h); a.hl = hl; a.h_off_q = L.kp128;
    a.counters = (unsigned*)(ws + w.off_cnt); a.n_counters = G;
    if (grid1 > 0) {
      int rc;
      if (gpw <= 1) rc = launch_phase1<1, 8>(a, grid1, st);
      else if (gpw <= 2) rc = launch_phase1<2, 8>(a, grid1, st);
      else rc = launch_phase1<4, 8>(a, grid1, st);
      if (rc) return rc;
    }
    Phase2Args b = {};
    b.h = a.h; b.T = T; b.d = dm; b.hl = hl; b.h_off_q = L.kp128; b.S = S;
    b.hv_down = (const u32x4_t*)(split + L.off_hv[2]);
    b.JBh = L.kp128 / 128;
    b.q_down = (const u32x4_t*)(split + L.off_i4[2]);
    b.s_down = (const uint16_t*)(split + L.off_s4[2]);
    b.JBr = m > 0 ? L.jp128 / 128 : 0;
    b.jp128 = L.jp128;
    b.part = (float*)(ws + w.off_part);
    b.counters = (unsigned*)(ws + w.off_cnt);
    b.Y = ep.out_f32 ? (bf16_t*)((float*)Y + (int64_t)t0 * dm) : (bf16_t*)Y + (int64_t)t0 * dm;
    b.b2 = ep.b2; b.resid = ep.resid ? ep.resid + (int64_t)t0 * dm : nullptr; b.out_f32 = ep.out_f32;
    b.Yh = Y_heavy ? (bf16_t*)Y_heavy + (int64_t)t0 * dm : nullptr;
    b.Yr = Y_rem ? (bf16_t*)Y_rem + (int64_t)t0 * dm : nullptr;
    hipLaunchKernelGGL(int4_phase2_kernel, dim3(G, S), dim3(512), 0, st, b);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

}  // namespace ffsplit
