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

// ---------------------------------------------------------------- decode, phase 1
// h[t, j] = act(x_t . up_j [, x_t . gate_j]) for every heavy and remainder neuron.
// A workgroup of 8 wavefronts walks over neuron tiles; wavefront w owns the
// quantisation groups w*GPW .. w*GPW+GPW-1 of the reduction and keeps the tokens'
// activations for them in registers for the whole kernel; the 8 partial 16x16
// results are added in a fixed order through LDS.

struct Phase1Args {
  const bf16_t* X;      // [T, d]
  int T, d, G;
  int n_up;             // 1: GeLU(up)   2: silu(gate) * up
  const uint4* hv_up;   // heavy blocks
  const uint4* hv_gate;
  int n_htiles;
  const uint4* q_up;    // int4 blocks
  const uint4* q_gate;
  const uint16_t* s_up;
  const uint16_t* s_gate;
  int n_qtiles;
  float* h;             // [16, hl] fp32
  int hl, h_off_q;      // remainder neurons start at column h_off_q
};

template <int GPW>
__global__ void __launch_bounds__(512) int4_phase1_kernel(const Phase1Args p) {
  __shared__ float red[2][8][2][256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, q = lane >> 4;

  Frag xr[GPW][4];
  float xsum[GPW];
#pragma unroll
  for (int i = 0; i < GPW; ++i) {
    const int g = wave * GPW + i;
    float s = 0.f;
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (g < p.G && n < p.T) v = *(const uint4*)(p.X + (int64_t)n * p.d + g * 128 + 32 * st + 8 * q);
      xr[i][st].u = v;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s += __uint_as_float(xr[i][st].w[e] << 16);
        s += __uint_as_float(xr[i][st].w[e] & 0xffff0000u);
      }
    }
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    xsum[i] = s;
  }

  const int n_tiles = p.n_htiles + p.n_qtiles;
  int par = 0;
  for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x, par ^= 1) {
    f32x4_t au = {0.f, 0.f, 0.f, 0.f}, ag = {0.f, 0.f, 0.f, 0.f};
    int hcol;
    if (tile < p.n_htiles) {
      hcol = tile * 16;
#pragma unroll
      for (int i = 0; i < GPW; ++i) {
        const int g = wave * GPW + i;
        if (g >= p.G) continue;
        const int64_t base = (((int64_t)tile * p.G + g) * 4) * 64 + lane;
        Frag wu[4], wg[4];
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          wu[st].u = p.hv_up[base + st * 64];
          if (p.n_up == 2) wg[st].u = p.hv_gate[base + st * 64];
        }
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          au = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wu[st].v, xr[i][st].v, au, 0, 0, 0);
          if (p.n_up == 2) ag = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wg[st].v, xr[i][st].v, ag, 0, 0, 0);
        }
      }
    } else {
      const int qt = tile - p.n_htiles;
      hcol = p.h_off_q + qt * 16;
      uint4 wu[GPW], wg[GPW];
      uint2 su[GPW], sg[GPW];
#pragma unroll
      for (int i = 0; i < GPW; ++i) {
        const int g = wave * GPW + i;
        if (g >= p.G) continue;
        const int64_t blk = (int64_t)qt * p.G + g;
        wu[i] = p.q_up[blk * 64 + lane];
        su[i] = *(const uint2*)(p.s_up + blk * 16 + 4 * q);
        if (p.n_up == 2) {
          wg[i] = p.q_gate[blk * 64 + lane];
          sg[i] = *(const uint2*)(p.s_gate + blk * 16 + 4 * q);
        }
      }
#pragma unroll
      for (int i = 0; i < GPW; ++i) {
        const int g = wave * GPW + i;
        if (g >= p.G) continue;
        const float corr = 136.f * xsum[i];
        {
          f32x4_t raw = {0.f, 0.f, 0.f, 0.f};
          const uint32_t w4[4] = {wu[i].x, wu[i].y, wu[i].z, wu[i].w};
#pragma unroll
          for (int st = 0; st < 4; ++st)
            raw = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dequant8(w4[st]).v, xr[i][st].v, raw, 0, 0, 0);
          const uint16_t sb[4] = {(uint16_t)(su[i].x & 0xffff), (uint16_t)(su[i].x >> 16),
                                  (uint16_t)(su[i].y & 0xffff), (uint16_t)(su[i].y >> 16)};
#pragma unroll
          for (int r = 0; r < 4; ++r) au[r] = fmaf(half_bits_to_f32(sb[r]), raw[r] - corr, au[r]);
        }
        if (p.n_up == 2) {
          f32x4_t raw = {0.f, 0.f, 0.f, 0.f};
          const uint32_t w4[4] = {wg[i].x, wg[i].y, wg[i].z, wg[i].w};
#pragma unroll
          for (int st = 0; st < 4; ++st)
            raw = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dequant8(w4[st]).v, xr[i][st].v, raw, 0, 0, 0);
          const uint16_t sb[4] = {(uint16_t)(sg[i].x & 0xffff), (uint16_t)(sg[i].x >> 16),
                                  (uint16_t)(sg[i].y & 0xffff), (uint16_t)(sg[i].y >> 16)};
#pragma unroll
          for (int r = 0; r < 4; ++r) ag[r] = fmaf(half_bits_to_f32(sb[r]), raw[r] - corr, ag[r]);
        }
      }
    }
    // lane holds neurons 4 q + r (r = 0..3) of the tile for token n
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      red[par][wave][0][lane * 4 + r] = au[r];
      red[par][wave][1][lane * 4 + r] = ag[r];
    }
    __syncthreads();
    if (tid < 256) {
      float u = 0.f, g = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) {
        u += red[par][w][0][tid];
        g += red[par][w][1][tid];
      }
      const int l = tid >> 2, r = tid & 3;
      const int tok = l & 15, neuron = 4 * (l >> 4) + r;
      const float hv = p.n_up == 2 ? silu_f(g) * u : gelu_f(u);
      if (tok < p.T) p.h[(int64_t)tok * p.hl + hcol + neuron] = hv;
    }
  }
}

// ---------------------------------------------------------------- decode, phase 2
// y[t, c] = sum_j h[t, j] * down[j, c].  Workgroup (cg, split) owns 128 outputs c
// and a range of 128-neuron blocks; its 4 wavefronts take blocks round-robin and
// are added in a fixed order; per-split partial sums go to `part`.

struct Phase2Args {
  const float* h;        // [16, hl]
  int T, d, hl;
  int heavy;             // 1: bf16 heavy blocks, 0: int4 blocks
  const uint4* w;        // blocks
  const uint16_t* sc;    // int4: [cg][jp128] fp16
  int JB, jp128;         // neuron blocks of 128; scale row length
  int h_off;             // first h column of this part
  int n_split;
  float* part;           // [n_split, 16, d] fp32 (this part's slice)
};

__global__ void __launch_bounds__(256) int4_phase2_kernel(const Phase2Args p) {
  __shared__ float red[4][8][256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, q = lane >> 4;
  const int cg = blockIdx.x, sp = blockIdx.y;
  const int per = (p.JB + p.n_split - 1) / p.n_split;
  const int jb0 = sp * per, jb1 = min(p.JB, jb0 + per);

  f32x4_t acc[8];
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) acc[ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float hsum = 0.f;

  for (int jb = jb0 + wave; jb < jb1; jb += 4) {
    // activations of this block's 128 neurons for token n, scaled per neuron (int4)
    Frag hb[4];
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const int j = jb * 128 + 32 * st + 8 * q;
      float hv[8];
      if (n < p.T) {
        const float4 a = *(const float4*)(p.h + (int64_t)n * p.hl + p.h_off + j);
        const float4 b = *(const float4*)(p.h + (int64_t)n * p.hl + p.h_off + j + 4);
        hv[0] = a.x; hv[1] = a.y; hv[2] = a.z; hv[3] = a.w; hv[4] = b.x; hv[5] = b.y; hv[6] = b.z; hv[7] = b.w;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) hv[e] = 0.f;
      }
      if (!p.heavy) {
        const uint4 sv = *(const uint4*)(p.sc + (int64_t)cg * p.jp128 + j);
        const uint32_t s4[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          hv[2 * e] *= half_bits_to_f32((uint16_t)(s4[e] & 0xffff));
          hv[2 * e + 1] *= half_bits_to_f32((uint16_t)(s4[e] >> 16));
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        hb[st].w[e] = pack_bf16x2(hv[2 * e], hv[2 * e + 1]);
        hsum += __uint_as_float(hb[st].w[e] << 16) + __uint_as_float(hb[st].w[e] & 0xffff0000u);
      }
    }
    if (p.heavy) {
      const int64_t base = ((((int64_t)cg * p.JB + jb) * 8) * 4) * 64 + lane;
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        Frag w[4];
#pragma unroll
        for (int st = 0; st < 4; ++st) w[st].u = p.w[base + (ct * 4 + st) * 64];
#pragma unroll
        for (int st = 0; st < 4; ++st)
          acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[st].v, hb[st].v, acc[ct], 0, 0, 0);
      }
    } else {
      const int64_t base = (((int64_t)cg * p.JB + jb) * 8) * 64 + lane;
      uint4 w[8];
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) w[ct] = p.w[base + ct * 64];
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const uint32_t w4[4] = {w[ct].x, w[ct].y, w[ct].z, w[ct].w};
#pragma unroll
        for (int st = 0; st < 4; ++st)
          acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dequant8(w4[st]).v, hb[st].v, acc[ct], 0, 0, 0);
      }
    }
  }
  if (!p.heavy) {
    hsum += __shfl_xor(hsum, 16);
    hsum += __shfl_xor(hsum, 32);
    const float corr = 136.f * hsum;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[ct][r] -= corr;
  }
#pragma unroll
  for (int ct = 0; ct < 8; ++ct)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][ct][lane * 4 + r] = acc[ct][r];
  __syncthreads();
  // 8 tiles x 256 values; thread handles value `tid` of every tile
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) {
    const float v = ((red[0][ct][tid] + red[1][ct][tid]) + red[2][ct][tid]) + red[3][ct][tid];
    const int l = tid >> 2, r = tid & 3;
    const int tok = l & 15, c = cg * 128 + ct * 16 + 4 * (l >> 4) + r;
    if (tok < p.T) p.part[((int64_t)sp * 16 + tok) * p.d + c] = v;
  }
}

// Y = bf16(sum of heavy partials + sum of remainder partials), fixed order
__global__ void int4_final_kernel(const float* part_h, int nh, const float* part_r, int nr, int T, int d,
                                  bf16_t* Y, bf16_t* Yh, bf16_t* Yr) {
  const int id = blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= T * d) return;
  const int t = id / d, c = id % d;
  float a = 0.f, b = 0.f;
  for (int s = 0; s < nh; ++s) a += part_h[((int64_t)s * 16 + t) * d + c];
  for (int s = 0; s < nr; ++s) b += part_r[((int64_t)s * 16 + t) * d + c];
  Y[id] = f32_to_bf16(a + b);
  if (Yh) Yh[id] = f32_to_bf16(a);
  if (Yr) Yr[id] = f32_to_bf16(b);
}

FwdWs make_fwd_ws(const ffsplit_desc_t& d, const Layout& L, int64_t T) {
  FwdWs w = {};
  const int m = d.d_ff - d.k;
  if (d.rem_kind == FFSPLIT_REM_INT4) {
    const int hl = L.kp128 + L.jp128;
    w.off_h = 0;
    size_t off = align256((size_t)16 * (hl > 0 ? hl : 1) * 4);
    const int JBh = L.kp128 / 128, JBr = m > 0 ? L.jp128 / 128 : 0;
    const int sh = (JBh + 1) / 2, sr = (JBr + 7) / 8;
    w.n_split = sh + sr;
    w.off_part = off;
    off += align256((size_t)(w.n_split > 0 ? w.n_split : 1) * 16 * d.d_model * 4);
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
  if (L.tiled && L.rp > 0 && L.mp > 0 && T > 0) {
    // split the long reduction of h2 * P2 until about two workgroups per CU exist
    const int tiles = (int)((T + 255) / 256) * ((L.rp + 127) / 128);
    int sp = 512 / (tiles > 0 ? tiles : 1);
    const int max_sp = L.mp / 256 > 0 ? L.mp / 256 : 1;   // keep >= 8 slabs of 32 per split
    if (sp > max_sp) sp = max_sp;
    if (sp > 16) sp = 16;
    if (sp < 1) sp = 1;
    w.g3_split = sp;
    if (sp > 1) off = align256(off + (size_t)sp * T * L.rp * 4);
  }
  w.total_bytes = off > 0 ? off : 256;
  return w;
}

template <int GPW>
static int launch_phase1(const Phase1Args& a, int grid, hipStream_t st) {
  hipLaunchKernelGGL(int4_phase1_kernel<GPW>, dim3(grid), dim3(512), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int int4_forward(const ffsplit_desc_t& d, const Layout& L, const FwdWs& w, const char* split, const void* X, int M,
                 void* Y, void* Y_heavy, void* Y_rem, char* ws, hipStream_t st) {
  const int m = d.d_ff - d.k, dm = d.d_model, G = L.groups;
  const int hl = L.kp128 + L.jp128;
  float* h = (float*)(ws + w.off_h);
  float* part = (float*)(ws + w.off_part);
  const int JBh = L.kp128 / 128, JBr = m > 0 ? L.jp128 / 128 : 0;
  const int sh = (JBh + 1) / 2, sr = (JBr + 7) / 8;
  const int gpw = (G + 7) / 8;
  if (gpw > 8) return -2;
  for (int t0 = 0; t0 < M; t0 += 16) {
    const int T = M - t0 < 16 ? M - t0 : 16;
    // h columns that no neuron writes (padding up to the 128-blocks) must read as zero
    if (launch_fill_zero(h, align256((size_t)16 * hl * 4), st)) return -1;
    Phase1Args a = {};
    a.X = (const bf16_t*)X + (int64_t)t0 * dm;
    a.T = T; a.d = dm; a.G = G; a.n_up = L.n_up;
    a.hv_up = (const uint4*)(split + L.off_hv[0]);
    a.hv_gate = (const uint4*)(split + L.off_hv[1]);
    a.n_htiles = L.kp / 16;
    a.q_up = (const uint4*)(split + L.off_i4[0]);
    a.q_gate = (const uint4*)(split + L.off_i4[1]);
    a.s_up = (const uint16_t*)(split + L.off_s4[0]);
    a.s_gate = (const uint16_t*)(split + L.off_s4[1]);
    a.n_qtiles = m > 0 ? L.jp16 / 16 : 0;
    a.h = h; a.hl = hl; a.h_off_q = L.kp128;
    const int n_tiles = a.n_htiles + a.n_qtiles;
    if (n_tiles > 0) {
      const int grid = n_tiles < 512 ? n_tiles : 512;
      int rc;
      if (gpw <= 1) rc = launch_phase1<1>(a, grid, st);
      else if (gpw <= 2) rc = launch_phase1<2>(a, grid, st);
      else if (gpw <= 4) rc = launch_phase1<4>(a, grid, st);
      else rc = launch_phase1<8>(a, grid, st);
      if (rc) return rc;
    }
    Phase2Args b = {};
    b.h = h; b.T = T; b.d = dm; b.hl = hl;
    if (JBh > 0) {
      b.heavy = 1; b.w = (const uint4*)(split + L.off_hv[2]); b.sc = nullptr; b.JB = JBh; b.jp128 = 0;
      b.h_off = 0; b.n_split = sh; b.part = part;
      hipLaunchKernelGGL(int4_phase2_kernel, dim3(G, sh), dim3(256), 0, st, b);
      if (hipGetLastError() != hipSuccess) return -1;
    }
    if (JBr > 0) {
      b.heavy = 0; b.w = (const uint4*)(split + L.off_i4[2]); b.sc = (const uint16_t*)(split + L.off_s4[2]);
      b.JB = JBr; b.jp128 = L.jp128; b.h_off = L.kp128; b.n_split = sr;
      b.part = part + (size_t)sh * 16 * dm;
      hipLaunchKernelGGL(int4_phase2_kernel, dim3(G, sr), dim3(256), 0, st, b);
      if (hipGetLastError() != hipSuccess) return -1;
    }
    const int n = T * dm;
    hipLaunchKernelGGL(int4_final_kernel, dim3((n + 255) / 256), dim3(256), 0, st, part, sh,
                       part + (size_t)sh * 16 * dm, sr, T, dm, (bf16_t*)Y + (int64_t)t0 * dm,
                       Y_heavy ? (bf16_t*)Y_heavy + (int64_t)t0 * dm : nullptr,
                       Y_rem ? (bf16_t*)Y_rem + (int64_t)t0 * dm : nullptr);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

}  // namespace ffsplit
