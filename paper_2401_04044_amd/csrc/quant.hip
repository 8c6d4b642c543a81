// The 8-bit heavy / 3-bit remainder split (Sec. 5.2, the setting used for the LLMs): build-time
// quantise-and-pack into the quantised tiled format (qformat.h), the unpack hook of the tests,
// and the expansion to a bf16 image in the DENSE layout for large batches.
//
// Quantisation groups run along d_model for every matrix, as for the int4 remainder: an up or
// gate column of a neuron has one scale per 128 inputs; a down row of a neuron has one scale
// per 128 outputs, so in the down matrices (rows = outputs, reduction over neurons) the scale
// changes with every reduction element and is constant over 128 consecutive rows.
#include "quant.h"
#include "prep.h"
#include "qformat.h"

namespace ffsplit {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

namespace {

// write the lane's 32 offset-binary codes u[t] into its place of a block
template <int BITS>
__device__ __forceinline__ void store_codes(char* block, int lane, const uint32_t u[32]) {
  if (BITS == 8) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      u32x4_t w;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t0 = 16 * h + 4 * i;   // operand block 2 h + (i >> 1), elements 4 (i & 1) ..
        w[i] = u[t0] | (u[t0 + 1] << 8) | (u[t0 + 2] << 16) | (u[t0 + 3] << 24);
      }
      *(u32x4_t*)(block + 1024 * h + lane * 16) = w;
    }
  } else {
    uint32_t lo[2] = {0, 0}, hi = 0;
#pragma unroll
    for (int t = 0; t < 32; ++t) {
      lo[t >> 4] |= (u[t] & 3u) << q_pos_lo(t);
      hi |= ((u[t] >> 2) & 1u) << q_pos_hi(t);
    }
    uint32_t* w = (uint32_t*)(block + lane * 12);
    w[0] = lo[0]; w[1] = lo[1]; w[2] = hi;
  }
}

// ---- up / gate: W [d, d_ff] bf16, rows of the packed matrix = neurons (SwiGLU: 32-row blocks
// alternate gate / up), one workgroup per (row block, group of 128 inputs)
struct PackUpArgs {
  const bf16_t* W1;
  const bf16_t* Wg;
  int d_ff, n_up, G;
  const int32_t* map;   // neuron position -> column
  int count;            // valid positions
  char* codes;
  uint16_t* scales;     // [row block][G][32]
};

template <int BITS>
__global__ void __launch_bounds__(256) pack_up_q_kernel(const PackUpArgs a) {
  __shared__ float tile[128][33];
  __shared__ float pm[8][32];
  __shared__ float sf[32];
  const int rb = blockIdx.x, g = blockIdx.y, tid = threadIdx.x;
  {
    const int r = tid & 31, kk0 = tid >> 5;
    const int rr = rb * 32 + r;
    const bool up = a.n_up == 2 ? ((rr >> 5) & 1) : true;
    const int n = a.n_up == 2 ? ((rr >> 6) * 32 + (rr & 31)) : rr;
    const bf16_t* W = up ? a.W1 : a.Wg;
    const int col = n < a.count ? a.map[n] : -1;
    float mx = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int kk = kk0 * 16 + i;
      const float v = col >= 0 ? bf16_to_f32(W[(int64_t)(g * 128 + kk) * a.d_ff + col]) : 0.f;
      tile[kk][r] = v;
      mx = fmaxf(mx, fabsf(v));
    }
    pm[kk0][r] = mx;
  }
  __syncthreads();
  if (tid < 32) {
    float m = 0.f;
#pragma unroll
    for (int p = 0; p < 8; ++p) m = fmaxf(m, pm[p][tid]);
    uint16_t bits;
    sf[tid] = q_scale(m, BITS, &bits);
    a.scales[((int64_t)rb * a.G + g) * 32 + tid] = bits;
  }
  __syncthreads();
  if (tid < 128) {
    const int b2 = tid >> 6, lane = tid & 63, r = lane & 31, c = lane >> 5;
    const float s = sf[r];
    uint32_t u[32];
#pragma unroll
    for (int t = 0; t < 32; ++t) u[t] = q_code(tile[64 * b2 + 16 * (t >> 3) + 8 * c + (t & 7)][r], s, BITS);
    char* block = a.codes + ((int64_t)rb * (a.G * 2) + 2 * g + b2) * (BITS == 8 ? 2048 : 768);
    store_codes<BITS>(block, lane, u);
  }
}

// ---- down: W2 [d_ff, d] bf16, rows of the packed matrix = outputs c, reduction over neuron
// positions; one workgroup per (128 outputs, 64 neurons)
struct PackDownArgs {
  const bf16_t* W2;
  int d;
  const int32_t* map;   // neuron position -> row of W2
  int count, Kp;        // valid / padded positions
  char* codes;
  uint16_t* scales;     // [d / 128][Kp]
};

template <int BITS>
__global__ void __launch_bounds__(256) pack_down_q_kernel(const PackDownArgs a) {
  __shared__ uint16_t tile[64][136];
  __shared__ float sf[64];
  const int cg = blockIdx.x, B = blockIdx.y, tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int jl = (tid >> 4) + 16 * i, chunk = tid & 15;
    const int p = B * 64 + jl;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (p < a.count) v = *(const uint4*)(a.W2 + (int64_t)a.map[p] * a.d + cg * 128 + chunk * 8);
    *(uint4*)&tile[jl][chunk * 8] = v;
  }
  __syncthreads();
  if (tid < 64) {
    float m = 0.f;
    for (int c = 0; c < 128; ++c) m = fmaxf(m, fabsf(bf16_to_f32(tile[tid][c])));
    uint16_t bits;
    sf[tid] = q_scale(m, BITS, &bits);
    a.scales[(int64_t)cg * a.Kp + B * 64 + tid] = bits;
  }
  __syncthreads();
  {
    const int rbl = tid >> 6, lane = tid & 63, r = lane & 31, c2 = lane >> 5;
    uint32_t u[32];
#pragma unroll
    for (int t = 0; t < 32; ++t) {
      const int jl = 16 * (t >> 3) + 8 * c2 + (t & 7);
      u[t] = q_code(bf16_to_f32(tile[jl][rbl * 32 + r]), sf[jl], BITS);
    }
    char* block = a.codes + ((int64_t)(cg * 4 + rbl) * (a.Kp / 64) + B) * (BITS == 8 ? 2048 : 768);
    store_codes<BITS>(block, lane, u);
  }
}

// ---- unpack hook: logical [n, d] codes and [n, G] scale bits
struct ExportArgs {
  const char* codes;
  const uint16_t* scales;
  int bits, down, n_up, up, G, d, Kp, n;
  int8_t* q_out;
  uint16_t* s_out;
};

__global__ void export_q_kernel(const ExportArgs a) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)a.n * a.d) return;
  const int p = (int)(id / a.d), c = (int)(id % a.d);
  int rb, r, B, rest, kblocks;
  uint16_t sbits;
  if (!a.down) {
    const int rr = a.n_up == 2 ? ((p >> 5) * 64 + (p & 31) + (a.up ? 32 : 0)) : p;
    rb = rr >> 5; r = rr & 31; B = c >> 6; rest = c & 63; kblocks = a.G * 2;
    sbits = a.scales[((int64_t)rb * a.G + (c >> 7)) * 32 + r];
  } else {
    rb = c >> 5; r = c & 31; B = p >> 6; rest = p & 63; kblocks = a.Kp / 64;
    sbits = a.scales[(int64_t)(c >> 7) * a.Kp + p];
  }
  const int j = rest >> 4, c2 = (rest >> 3) & 1, e = rest & 7, lane = 32 * c2 + r, t = 8 * j + e;
  const char* block = a.codes + ((int64_t)rb * kblocks + B) * (a.bits == 8 ? 2048 : 768);
  a.q_out[id] = (int8_t)(a.bits == 8 ? q_get(q_load8(block, lane), t) : q_get(q_load3(block, lane), t));
  if ((c & 127) == 0) a.s_out[(int64_t)p * a.G + (c >> 7)] = sbits;
}

// ---- expansion to the DENSE image (tiled bf16): one thread per 16-byte chunk of the image
struct ExpandQArgs {
  const char* codes[4];
  const uint16_t* scales[4];
  int n_up, G, d, kp, mp;
  int64_t n_chunks;
  u32x4_t* out;
};

__device__ __forceinline__ u32x4_t expand_chunk(const char* block, int bits, int lane, int j, const float s[8]) {
  if (bits == 8) {
    const QPacked<8> p = q_load8(block, lane);
    u32x4_t o;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      o[i] = pack_bf16x2((float)q_get(p, 8 * j + 2 * i) * s[2 * i], (float)q_get(p, 8 * j + 2 * i + 1) * s[2 * i + 1]);
    return o;
  }
  const QPacked<3> p = q_load3(block, lane);
  u32x4_t o;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    o[i] = pack_bf16x2((float)q_get(p, 8 * j + 2 * i) * s[2 * i], (float)q_get(p, 8 * j + 2 * i + 1) * s[2 * i + 1]);
  return o;
}

// B1t image [n_up (kp + mp), d]
__global__ void __launch_bounds__(256) expand_up_q_kernel(const ExpandQArgs a) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= a.n_chunks) return;
  const int lane = (int)(id & 63);
  const int64_t blk = id >> 6;
  const int kbs = a.d / 16;
  const int rb = (int)(blk / kbs), kb = (int)(blk % kbs);
  const int heavy_rb = a.n_up * a.kp / 32;
  const int mat = rb < heavy_rb ? 0 : 1;
  const int rbm = mat ? rb - heavy_rb : rb;
  const float sc = q_half(a.scales[mat][((int64_t)rbm * a.G + (kb >> 3)) * 32 + (lane & 31)]);
  const float s[8] = {sc, sc, sc, sc, sc, sc, sc, sc};
  const int bits = mat ? 3 : 8;
  const char* block = a.codes[mat] + ((int64_t)rbm * (a.G * 2) + (kb >> 2)) * (bits == 8 ? 2048 : 768);
  a.out[id] = expand_chunk(block, bits, lane, kb & 3, s);
}

// B4t image [d, kp + mp]
__global__ void __launch_bounds__(256) expand_down_q_kernel(const ExpandQArgs a) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= a.n_chunks) return;
  const int lane = (int)(id & 63);
  const int64_t blk = id >> 6;
  const int kbs = (a.kp + a.mp) / 16;
  const int rb = (int)(blk / kbs), kb = (int)(blk % kbs);
  const int mat = kb < a.kp / 16 ? 2 : 3;
  const int kbm = mat == 3 ? kb - a.kp / 16 : kb;
  const int Kp = mat == 3 ? a.mp : a.kp;
  const int p0 = kbm * 16 + 8 * (lane >> 5);
  const uint4 sb = *(const uint4*)(a.scales[mat] + (int64_t)(rb >> 2) * Kp + p0);
  const uint32_t sw[4] = {sb.x, sb.y, sb.z, sb.w};
  float s[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    s[2 * i] = q_half((uint16_t)(sw[i] & 0xffffu));
    s[2 * i + 1] = q_half((uint16_t)(sw[i] >> 16));
  }
  const int bits = mat == 3 ? 3 : 8;
  const char* block = a.codes[mat] + ((int64_t)rb * (Kp / 64) + (kbm >> 2)) * (bits == 8 ? 2048 : 768);
  a.out[id] = expand_chunk(block, bits, lane, kbm & 3, s);
}

}  // namespace

int launch_w3h8_pack(const ffsplit_desc_t& d, const Layout& L, const void* W1, const void* Wg, const void* W2,
                     const int32_t* rest, const int32_t* idx, char* split, hipStream_t st) {
  const int m = d.d_ff - d.k;
  for (int i = 0; i < 2; ++i) {   // 0 heavy (8 bits), 1 remainder (3 bits)
    const int count = i ? m : d.k, Kp = i ? L.mp : L.kp;
    if (count <= 0) continue;
    const int32_t* map = i ? rest : idx;
    PackUpArgs u = {};
    u.W1 = (const bf16_t*)W1; u.Wg = (const bf16_t*)Wg; u.d_ff = d.d_ff; u.n_up = L.n_up; u.G = L.groups;
    u.map = map; u.count = count;
    u.codes = split + L.off_qc[i]; u.scales = (uint16_t*)(split + L.off_qs[i]);
    const dim3 gu(L.n_up * Kp / 32, L.groups);
    if (i) hipLaunchKernelGGL(pack_up_q_kernel<3>, gu, dim3(256), 0, st, u);
    else hipLaunchKernelGGL(pack_up_q_kernel<8>, gu, dim3(256), 0, st, u);
    if (hipGetLastError() != hipSuccess) return -1;
    PackDownArgs w = {};
    w.W2 = (const bf16_t*)W2; w.d = d.d_model; w.map = map; w.count = count; w.Kp = Kp;
    w.codes = split + L.off_qc[2 + i]; w.scales = (uint16_t*)(split + L.off_qs[2 + i]);
    const dim3 gd(d.d_model / 128, Kp / 64);
    if (i) hipLaunchKernelGGL(pack_down_q_kernel<3>, gd, dim3(256), 0, st, w);
    else hipLaunchKernelGGL(pack_down_q_kernel<8>, gd, dim3(256), 0, st, w);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

int launch_w3h8_export(const ffsplit_desc_t& d, const Layout& L, const char* split, int what, int8_t* q_out,
                       uint16_t* s_out, hipStream_t st) {
  const bool heavy = what >= 3;
  const int w3 = what % 3;
  const int n = heavy ? d.k : d.d_ff - d.k;
  if (n <= 0) return 0;
  const int mat = (w3 == 2 ? 2 : 0) + (heavy ? 0 : 1);
  ExportArgs a = {};
  a.codes = split + L.off_qc[mat]; a.scales = (const uint16_t*)(split + L.off_qs[mat]);
  a.bits = heavy ? 8 : 3; a.down = w3 == 2; a.n_up = L.n_up; a.up = w3 == 0; a.G = L.groups; a.d = d.d_model;
  a.Kp = heavy ? L.kp : L.mp; a.n = n; a.q_out = q_out; a.s_out = s_out;
  const int64_t total = (int64_t)n * d.d_model;
  hipLaunchKernelGGL(export_q_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_w3h8_expand(const ffsplit_desc_t& d, const Layout& L, const Layout& LD, const char* split, char* image,
                       hipStream_t st) {
  if (!LD.tiled || LD.dk != d.d_model || LD.dn != d.d_model || LD.kp != L.kp || LD.mp != L.mp) return -1;
  ExpandQArgs a = {};
  for (int i = 0; i < 4; ++i) {
    a.codes[i] = split + L.off_qc[i];
    a.scales[i] = (const uint16_t*)(split + L.off_qs[i]);
  }
  a.n_up = L.n_up; a.G = L.groups; a.d = d.d_model; a.kp = L.kp; a.mp = L.mp;
  if (LD.n1 > 0) {
    a.n_chunks = (int64_t)LD.n1 * d.d_model / 8;
    a.out = (u32x4_t*)(image + LD.off_b1);
    hipLaunchKernelGGL(expand_up_q_kernel, dim3((unsigned)((a.n_chunks + 255) / 256)), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  if (LD.k4 > 0) {
    a.n_chunks = (int64_t)LD.dn * LD.k4 / 8;
    a.out = (u32x4_t*)(image + LD.off_b4);
    hipLaunchKernelGGL(expand_down_q_kernel, dim3((unsigned)((a.n_chunks + 255) / 256)), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

int w3h8_forward_small(const ffsplit_desc_t& d, const Layout& L, const FwdWs& w, const char* split, const void* X,
                       int M, void* Y, void* Y_heavy, void* Y_rem, const Epilogue& ep, char* ws, hipStream_t st) {
  const int dm = d.d_model;
  const int act = d.act == FFSPLIT_ACT_SWIGLU ? ACT_GLU : ACT_GELU;
  char* cat = ws + w.off_cat;                  // [32, k4] tiled fp16: activated heavy | remainder neurons
  float* part = (float*)(ws + w.off_kpart);
  const size_t esz = 2;
  auto koff = [&](int col) { return (size_t)(col / 16) * 1024; };
  // up / gate product, heavy rows (8 bits) then remainder rows (3 bits): act(X W) into cat
  {
    GemmArgs g8 = {}, g3 = {};
    g8.A = X; g8.lda = dm; g8.M = M; g8.N = L.n_up * L.kp; g8.K = dm;
    g3 = g8; g3.N = L.n_up * L.mp;
    SkinnyQ q8 = {split + L.off_qc[0], split + L.off_qs[0], 8, 0, L.groups, 0};
    SkinnyQ q3 = {split + L.off_qc[1], split + L.off_qs[1], 3, 0, L.groups, 0};
    int S[2];
    if (launch_skinny_q_pair(g8, q8, g3, q3, part, S, st)) return -1;
    GemmArgs g = g8;
    g.N = L.n_up * L.k4; g.act_cols = g.N; g.split_col = L.k4;
    g.C0 = cat; g.ldc0 = L.k4; g.c0_tiled = 1;
    if (g.N > 0 && launch_skinny_reduce2(g, act, part, S[0], L.n_up * L.kp / 32, S[1], 1, st)) return -1;
  }
  // down product: both segments of the reduction stream into partial tiles, one sum (Eq. 2's
  // addition happens in fp32, one rounding)
  GemmArgs g = {};
  g.M = M; g.N = dm; g.lda = L.k4; g.a_tiled = 1;
  g.split_col = dm; g.ldc0 = dm; g.n_store = dm;
  int S[2] = {0, 0};
  {
    GemmArgs g8 = g, g3 = g;
    g8.A = cat; g8.K = L.kp;
    g3.A = cat + koff(L.kp); g3.K = L.mp;
    SkinnyQ q8 = {split + L.off_qc[2], split + L.off_qs[2], 8, 1, L.groups, L.kp};
    SkinnyQ q3 = {split + L.off_qc[3], split + L.off_qs[3], 3, 1, L.groups, L.mp};
    if (launch_skinny_q_pair(g8, q8, g3, q3, part, S, st)) return -1;
  }
  const size_t seg = (size_t)S[0] * (dm / 32) * 1024;   // floats of the heavy segment's tiles
  auto emit = [&](void* out, const float* p0, int n) -> int {
    if (!out) return 0;
    if (n == 0) return launch_fill_zero(out, (size_t)M * dm * esz, st);
    g.C0 = out;
    return launch_skinny_reduce(g, ACT_NONE, p0, n, 0, st);
  };
  // (output bias, residual stream and an fp32 destination apply to Y only)
  g.bias = ep.b2; g.bias_cols = ep.b2 ? dm : 0; g.resid = ep.resid; g.ldr = dm; g.out_f32 = ep.out_f32;
  if (S[0] + S[1] == 0 && (ep.b2 || ep.resid || ep.out_f32)) return -2;
  if (emit(Y, part, S[0] + S[1])) return -1;
  g.bias = nullptr; g.bias_cols = 0; g.resid = nullptr; g.out_f32 = 0;
  if (emit(Y_heavy, part, S[0])) return -1;
  if (emit(Y_rem, part + seg, S[1])) return -1;
  return 0;
}

}  // namespace ffsplit
