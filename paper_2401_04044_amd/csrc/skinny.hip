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
#include "layout.h"
#include "qformat.h"

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
  int n_tb;           // 32-token blocks of the activations (at most NT of the kernel)
  float* part;        // [n_split][n_rb][NT][4][64] float4: accumulator order
};

template <bool A_TILED, int NT>
__global__ void __launch_bounds__(256) skinny_stream_kernel(const SkinnyArgs p) {
  constexpr int U = SK_U;   // blocks per register group
  const int lane = threadIdx.x & 63;
  const int task = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (task >= p.n_rb * p.n_split) return;
  const int rb = task % p.n_rb, sp = task / p.n_rb;
  const int kb_total = (p.K + 15) / 16;
  const int kb0 = sp * p.kb_per;
  const int kb1 = min(kb_total, kb0 + p.kb_per);
  const int kb_last = kb1 - 1;

  const char* wbase = (const char*)p.Bt + ((int64_t)rb * (p.ldb / 16) * 64 + lane) * 16;
  // one activation base per block of 32 tokens (a block past the batch repeats the last one;
  // its results are never read)
  const char* abase[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int tb = min(t, p.n_tb - 1);
    abase[t] = (const char*)((p.A1 != nullptr && (rb & 1)) ? p.A1 : p.A);
    if (A_TILED) {
      abase[t] += ((int64_t)tb * (p.lda / 16) * 64 + lane) * 16;
    } else {
      const int row = min(tb * 32 + (lane & 31), p.M - 1);
      abase[t] += ((int64_t)row * p.lda + (lane >> 5) * 8) * 2;
    }
  }
  // block kb of the weights / of the activations; past the range: the last block again (its
  // product is masked out below), so that the loads stay unconditional
  auto wload = [&](int kb) { return *(const u32x4_t*)(wbase + (int64_t)min(kb, kb_last) * 1024); };
  auto aload = [&](int t, int kb) {
    const int k = min(kb, kb_last);
    if (A_TILED) return *(const u32x4_t*)(abase[t] + (int64_t)k * 1024);
    // row-major: a chunk past K (K is a multiple of 8) reads the row's first chunk instead;
    // the weights are zero there
    const int col = k * 16 + (lane >> 5) * 8;
    return *(const u32x4_t*)(abase[t] + (col < p.K ? (int64_t)k * 32 : -(int64_t)((lane >> 5) * 16)));
  };

  f32x16_t acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  u32x4_t w0[U], a0[NT][U], w1[U], a1[NT][U];
  auto load = [&](u32x4_t* w, u32x4_t (*a)[U], int kb) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      w[u] = wload(kb + u);
#pragma unroll
      for (int t = 0; t < NT; ++t) a[t][u] = aload(t, kb + u);
    }
  };
  auto compute = [&](const u32x4_t* w, u32x4_t (*a)[U], int kb) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      SFrag wf;
      wf.u = w[u];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        SFrag af;
        af.u = (kb + u < kb1) ? a[t][u] : u32x4_t{0, 0, 0, 0};
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, af.v, acc[t], 0, 0, 0);
      }
    }
  };
  if (kb0 < kb1) {
    load(w0, a0, kb0);
    for (int kb = kb0; kb < kb1; kb += 2 * U) {
      load(w1, a1, kb + U);
      if (NT > 1) __builtin_amdgcn_sched_barrier(0);   // keep the batch of loads ahead of the arithmetic
      compute(w0, a0, kb);
      if (NT > 1) __builtin_amdgcn_sched_barrier(0);
      load(w0, a0, kb + 2 * U);
      if (NT > 1) __builtin_amdgcn_sched_barrier(0);
      compute(w1, a1, kb + U);
      if (NT > 1) __builtin_amdgcn_sched_barrier(0);
    }
  }
  // lane: row (token) = lane & 31; columns 8 g + 4 (lane >> 5) + 0..3 of the block in acc[4 g ..]
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    float4* dst = (float4*)p.part + ((int64_t)((sp * p.n_rb + rb) * NT + t) * 4) * 64 + lane;
#pragma unroll
    for (int g = 0; g < 4; ++g)
      dst[g * 64] = make_float4(acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]);
  }
}

// The same product with the weights in the quantised tiled format (32 x 64 blocks of 8- or
// 3-bit codes plus fp16 group scales; qformat.h).  The packed blocks are the only traffic that
// comes from HBM; they are unpacked in the integer domain: a shift, a rotate and two and-or
// per operand register give the pair (magic + u) directly.
//   UP    (one scale per row and 128 reduction elements; activations = the caller's bf16 X):
//         the unscaled codes go through the MFMA, one group of 128 at a time, and the group's
//         fp32 result is scaled per row afterwards.  3 bits: operands are the bf16 values
//         128 + u.  8 bits: the codes do not fit a bf16 mantissa; X is converted to fp16 (exact)
//         and the operands are the fp16 values 1024 + u.
//   DOWN  (one scale per reduction element and 128 rows; activations fp16, written by the UP
//         products' reduce step): the scale multiplies the activations (one packed multiply per
//         register, shared by the row blocks of the group) and the operands are the fp16 values
//         1024 + u.
//   In both, the constant 128 + 4, 1024 + 4 or 1024 + 128 leaves through a second MFMA per
//   operand block whose left operand holds the negated constant in every row.
// Work split: a workgroup of four wavefronts owns RB adjacent row blocks (they share the
// activation blocks, and for DOWN the scales) over one range of the reduction; the wavefronts
// take a quarter of the range each and add their accumulators through LDS in a fixed order.
// A wavefront requests the packed weights of up to SKQ_UNITS units (its whole share at the
// usual shapes) in one batch, so that they cost one round trip to memory, and then the
// activations and scales (cache resident) unit by unit, one unit ahead of the arithmetic.
struct SkinnyQArgs {
  const void* A;
  int64_t lda;
  int M, n_rb, n_split, nu_total, nu_per, slot0;   // units: UP groups of two blocks, DOWN blocks
  int rb_out0, n_rb_part;                          // partial tiles: first row block, row blocks per range
  const char* codes;
  const uint16_t* scales;
  int G, Kp;
  float* part;
};

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
union QFrag {
  u32x4_t u;
  bf16x8_t b;
  f16x8_t h;
};
union H2 {
  uint32_t u;
  f16x2_t h;
};

// Units whose weights a wavefront holds at once, and row blocks per workgroup of the 3-bit parts.
// Both are set by registers: at most 168 per lane keeps three workgroups per CU resident, which
// matters more here than sharing the activation loads among more row blocks (measured: four
// units and four row blocks, two workgroups per CU, 47 us per step at the Llama shape against 41.5).
constexpr int SKQ_UNITS = 2;
constexpr int SKQ_RB_UP3 = 2, SKQ_RB_DOWN3 = 2;

// row blocks per workgroup (they share the activation blocks and, for DOWN, the scales)
constexpr int skq_rb(int bits, bool down) { return bits == 3 ? (down ? SKQ_RB_DOWN3 : SKQ_RB_UP3) : (down ? 2 : 1); }

template <int BITS, bool DOWN>
struct QShape {
  static constexpr int RB = skq_rb(BITS, DOWN);
  static constexpr int UB = DOWN ? 1 : 2;                                  // blocks per unit
};

template <int BITS, bool DOWN>
struct QWts {
  QPacked<BITS> w[QShape<BITS, DOWN>::RB][QShape<BITS, DOWN>::UB];
};

template <int BITS, bool DOWN>
struct QAct {
  u32x4_t a[QShape<BITS, DOWN>::UB * 4];
  u32x4_t sd[DOWN ? 4 : 1];                                  // DOWN: scale pairs of the block's 64 elements
  u32x2_t su[DOWN ? 1 : QShape<BITS, DOWN>::RB][4];          // UP: the lane's 16 row scales per row block
};

template <int BITS, bool DOWN>
__device__ __forceinline__ void skinny_q_body(const SkinnyQArgs& p, int wg, float* red_mem) {
  constexpr int RB = QShape<BITS, DOWN>::RB, UB = QShape<BITS, DOWN>::UB;
  constexpr int BB = BITS == 8 ? 2048 : 768;
  constexpr bool F16 = DOWN || BITS == 8;                    // fp16 MFMA
  float (*red)[RB][16][64] = (float (*)[RB][16][64])red_mem;   // [4][RB][16][64]
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_rbg = p.n_rb / RB;
  const int rb = (wg % n_rbg) * RB, sp = wg / n_rbg;
  const int U0 = sp * p.nu_per;
  const int U1 = min(p.nu_total, U0 + p.nu_per);             // U0 < U1 by construction of the grid
  const int per = (U1 - U0 + 3) / 4;
  const int u0 = U0 + wave * per;
  const int u1 = min(U1, u0 + per);                          // may be empty: the wavefront then adds zeros
  const int r = lane & 31, c2 = lane >> 5;

  const char* wbase = p.codes + (int64_t)rb * p.nu_total * UB * BB;
  const int64_t wrow = (int64_t)p.nu_total * UB * BB;        // bytes from one row block to the next
  const char* abase = (const char*)p.A;
  if (DOWN) abase += (int64_t)lane * 16;                              // tiled, one row block
  else abase += ((int64_t)min(r, p.M - 1) * p.lda + c2 * 8) * 2;      // the caller's row-major X

  // (a unit past the range reads some valid unit of it and is not computed)
  auto load_w = [&](QWts<BITS, DOWN>& q, int u) {
    const int uc = max(U0, min(u, U1 - 1));
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
      for (int x = 0; x < UB; ++x) {
        const char* blk = wbase + i * wrow + (int64_t)(uc * UB + x) * BB;
        if constexpr (BITS == 8) q.w[i][x] = q_load8(blk, lane);
        else q.w[i][x] = q_load3(blk, lane);
      }
  };
  auto load_a = [&](QAct<BITS, DOWN>& q, int u) {
    const int uc = max(U0, min(u, U1 - 1));
#pragma unroll
    for (int kb = 0; kb < UB * 4; ++kb)
      q.a[kb] = *(const u32x4_t*)(abase + (int64_t)(uc * UB * 4 + kb) * (DOWN ? 1024 : 32));
    if constexpr (DOWN) {
      const uint16_t* sb = p.scales + (int64_t)(rb >> 2) * p.Kp + uc * 64 + 8 * c2;
#pragma unroll
      for (int j = 0; j < 4; ++j) q.sd[j] = *(const u32x4_t*)(sb + 16 * j);
    } else {
      // rows 8 g + 4 c2 + i of a row block live in accumulator registers 4 g + i
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        const uint16_t* sb = p.scales + ((int64_t)(rb + i) * p.G + uc) * 32 + 4 * c2;
#pragma unroll
        for (int g = 0; g < 4; ++g) q.su[i][g] = *(const u32x2_t*)(sb + 8 * g);
      }
    }
  };

  const f32x16_t zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  f32x16_t tot[RB];
#pragma unroll
  for (int i = 0; i < RB; ++i) tot[i] = zero;

  auto compute = [&](const QWts<BITS, DOWN>& qw, const QAct<BITS, DOWN>& q) {
    QFrag a[UB * 4];
#pragma unroll
    for (int kb = 0; kb < UB * 4; ++kb) {
      a[kb].u = q.a[kb];
      if constexpr (!DOWN && BITS == 8) {
        // bf16 -> fp16: eight significant bits, exact (round toward zero never rounds)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const auto h = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(a[kb].u[i] << 16),
                                                    __uint_as_float(a[kb].u[i] & 0xffff0000u));
          uint32_t hb;
          __builtin_memcpy(&hb, &h, 4);
          a[kb].u[i] = hb;
        }
      }
    }
    // The unpacked operands are the integers magic + u (u the offset-binary code); the constant
    // magic + 2^(bits-1) is removed by a second MFMA whose left operand is that constant,
    // negated, in every row: the vector ALU, which bounds these kernels, only unpacks.
    QFrag negc;
    {
      const uint32_t c = F16 ? (BITS == 8 ? 0xE480E480u /* -1152 */ : 0xE404E404u /* -1028 */) : 0xC304C304u /* bf16 -132 */;
      negc.u = u32x4_t{c, c, c, c};
    }
    if constexpr (DOWN) {
      // the scale depends on the reduction element (and the group of 128 rows, which the RB row
      // blocks share): it multiplies the activations, one packed multiply per register
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          H2 v, s2;
          v.u = a[j].u[i];
          s2.u = q.sd[j][i];
          v.h = v.h * s2.h;
          a[j].u[i] = v.u;
        }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int rbi = 0; rbi < RB; ++rbi) {
          QFrag wf;
#pragma unroll
          for (int i = 0; i < 4; ++i) wf.u[i] = q_pair(qw.w[rbi][0], j, i, BITS == 8 ? 0x64646464u : 0x64006400u);
          tot[rbi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf.h, a[j].h, tot[rbi], 0, 0, 0);
        }
#pragma unroll
        for (int rbi = 0; rbi < RB; ++rbi)
          tot[rbi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(negc.h, a[j].h, tot[rbi], 0, 0, 0);
      }
    } else {
      f32x16_t ag[RB];
#pragma unroll
      for (int i = 0; i < RB; ++i) ag[i] = zero;
#pragma unroll
      for (int kb = 0; kb < 8; ++kb) {
#pragma unroll
        for (int rbi = 0; rbi < RB; ++rbi) {
          QFrag wf;
#pragma unroll
          for (int i = 0; i < 4; ++i) wf.u[i] = q_pair(qw.w[rbi][kb >> 2], kb & 3, i, BITS == 8 ? 0x64646464u : 0x43004300u);
          if constexpr (F16) ag[rbi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf.h, a[kb].h, ag[rbi], 0, 0, 0);
          else ag[rbi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.b, a[kb].b, ag[rbi], 0, 0, 0);
        }
#pragma unroll
        for (int rbi = 0; rbi < RB; ++rbi) {
          if constexpr (F16) ag[rbi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(negc.h, a[kb].h, ag[rbi], 0, 0, 0);
          else ag[rbi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(negc.b, a[kb].b, ag[rbi], 0, 0, 0);
        }
      }
      // the group's integer dot products times the rows' scales for this group
#pragma unroll
      for (int rbi = 0; rbi < RB; ++rbi)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const u32x2_t sc = q.su[rbi][g];
          const float s4[4] = {q_half((uint16_t)(sc[0] & 0xffffu)), q_half((uint16_t)(sc[0] >> 16)),
                               q_half((uint16_t)(sc[1] & 0xffffu)), q_half((uint16_t)(sc[1] >> 16))};
#pragma unroll
          for (int i = 0; i < 4; ++i) tot[rbi][4 * g + i] = fmaf(s4[i], ag[rbi][4 * g + i], tot[rbi][4 * g + i]);
        }
    }
  };

  for (int ub = u0; ub < u1; ub += SKQ_UNITS) {
    QWts<BITS, DOWN> qw[SKQ_UNITS];
    QAct<BITS, DOWN> qa[2];
#pragma unroll
    for (int i = 0; i < SKQ_UNITS; ++i) load_w(qw[i], ub + i);
    load_a(qa[0], ub);
#pragma unroll
    for (int i = 0; i < SKQ_UNITS; ++i) {
      // (the scheduling barriers keep each batch of loads ahead of the arithmetic of the unit before)
      if (i + 1 < SKQ_UNITS) load_a(qa[(i + 1) & 1], ub + i + 1);
      __builtin_amdgcn_sched_barrier(0);
      if (ub + i < u1) compute(qw[i], qa[i & 1]);   // (wavefront-uniform)
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // fixed-order sum over the four wavefronts; wavefront w finishes accumulator registers 4 w ..
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave][i][v][lane] = tot[i][v];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    float o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      o[e] = red[0][i][4 * wave + e][lane];
#pragma unroll
      for (int w = 1; w < 4; ++w) o[e] += red[w][i][4 * wave + e][lane];
    }
    float4* dst = (float4*)p.part + ((int64_t)((p.slot0 + sp) * p.n_rb_part + p.rb_out0 + rb + i) * 4 + wave) * 64 + lane;
    *dst = make_float4(o[0], o[1], o[2], o[3]);
  }
}

// One launch for the 8-bit and the 3-bit part of a product: workgroups [0, wg8) take the
// first, the rest the second.
struct SkinnyQ2Args {
  SkinnyQArgs s8, s3;
  int wg8;
};

template <bool DOWN>
__global__ void __launch_bounds__(256) skinny_stream_q2_kernel(const SkinnyQ2Args p) {
  extern __shared__ float red_mem[];
  if ((int)blockIdx.x < p.wg8) skinny_q_body<8, DOWN>(p.s8, (int)blockIdx.x, red_mem);
  else skinny_q_body<3, DOWN>(p.s3, (int)blockIdx.x - p.wg8, red_mem);
}

__device__ __forceinline__ float sk_silu(float z) { return silu_fast(z); }   // exp2 and rcp: no division sequence

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
  int f16_out;   // destinations hold fp16 (saturating) instead of bf16
  int rb_split, n_split_b;   // row blocks from rb_split on have n_split_b ranges
  int n_tb, nt;              // 32-token blocks to write / token blocks per row block in part
  const float* bias;         // as in GemmArgs
  int bias_cols;
  const float* resid;
  int64_t ldr;
  int out_f32;
};

__device__ __forceinline__ uint32_t pack_f16x2_sat(float lo, float hi) {
  H2 v;
  v.h = f16x2_t{(_Float16)fminf(fmaxf(lo, -65504.f), 65504.f), (_Float16)fminf(fmaxf(hi, -65504.f), 65504.f)};
  return v.u;
}

// Activation and store of four consecutive output columns (registers 4 g .. 4 g + 3 of row
// block rb, token row lane & 31): v the block's sums, u the up block's sums for a (gate, up) pair.
__device__ __forceinline__ void sk_emit(const SkinnyReduceArgs& p, int rb, int tb, int g, int lane, float v[4],
                                        const float u[4]) {
  const int cb = rb * 32;
  const bool act_here = cb < p.act_cols;
  const bool glu = p.act == ACT_GLU;
  int oc = cb;
  if (glu) oc = act_here ? cb / 2 : cb - p.act_cols / 2;
  {
    // a neuron's bias (GEMM column cb + 8 g + 4 (lane >> 5) + e), before the activation
    const int c = cb + 8 * g + 4 * (lane >> 5);
    if (!glu && p.bias != nullptr && c + 3 < p.bias_cols) {
      const float4 b4 = *(const float4*)(p.bias + c);
      v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
    }
  }
  if (act_here) {
    if (glu) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = sk_silu(v[e]) * u[e];
    } else if (p.act == ACT_GELU) {
#pragma unroll
      // the bf16 path's GeLU (common.h); erff here costs the kernels that inline this 60 registers per
      // lane and with them a workgroup per CU
      for (int e = 0; e < 4; ++e) v[e] = gelu_fast(v[e]);
    }
  }
  const int row = tb * 32 + (lane & 31);
  const int col0 = oc + 8 * g + 4 * (lane >> 5);   // first of this thread's four output columns
  char* base;
  int64_t ld;
  int col, tiled;
  const bool to_c0 = col0 < p.split_col;
  if (to_c0) { base = (char*)p.C0; ld = p.ldc0; col = col0; tiled = p.c0_tiled; }
  else { base = (char*)p.C1; ld = p.ldc1; col = col0 - p.split_col; tiled = p.c1_tiled; }
  if (to_c0 && !tiled && row < p.M && col < p.n_store) {
    if (p.resid != nullptr) {
      const float4 r4 = *(const float4*)(p.resid + (int64_t)row * p.ldr + col);
      v[0] += r4.x; v[1] += r4.y; v[2] += r4.z; v[3] += r4.w;
    }
    if (p.out_f32) {
      *(float4*)((float*)base + (int64_t)row * ld + col) = make_float4(v[0], v[1], v[2], v[3]);
      return;
    }
  }
  const uint2 val = p.f16_out ? make_uint2(pack_f16x2_sat(v[0], v[1]), pack_f16x2_sat(v[2], v[3]))
                              : make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
  if (tiled) {
    // (rows past M in the last 32-row block hold repeats of row M - 1, finite)
    const int64_t chunk = ((int64_t)tb * (ld / 16) + col / 16) * 64 + ((col >> 3) & 1) * 32 + (lane & 31);
    *(uint2*)(base + chunk * 16 + (col & 7) * 2) = val;
  } else if (row < p.M && col < p.n_store) {
    *(uint2*)(base + ((int64_t)row * ld + col) * 2) = val;
  }
}

__global__ void __launch_bounds__(256) skinny_reduce_kernel(const SkinnyReduceArgs p) {
  const int id = blockIdx.x * 256 + threadIdx.x;
  if (id >= p.n_rb * p.n_tb * 256) return;
  const int rb = (id >> 8) / p.n_tb, tb = (id >> 8) % p.n_tb, g = (id >> 6) & 3, lane = id & 63;
  const bool pair = p.act == ACT_GLU && rb * 32 < p.act_cols;
  if (pair && (rb & 1)) return;   // the pair is written from its gate block
  auto sum_block = [&](int b) {
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    const float4* src = (const float4*)p.part + (((int64_t)b * p.nt + tb) * 4 + g) * 64 + lane;
    // eight independent loads at a time, added in range order (24 at a time, all ranges of the
    // usual products in one round trip, measured slower: 5.9 vs 4.3 us, and 8.4 vs 5.0 us where
    // there are few ranges and most of the 24 were repeats)
    const int64_t step = (int64_t)p.n_rb * p.nt * 256;
    const int ns = b < p.rb_split ? p.n_split : p.n_split_b;
    constexpr int NB = 8;
    for (int sp = 0; sp < ns; sp += NB) {
      float4 v[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) v[u] = src[(int64_t)min(sp + u, ns - 1) * step];
#pragma unroll
      for (int u = 0; u < NB; ++u)
        if (sp + u < ns) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
    return s;
  };
  const float4 z0 = sum_block(rb);
  float v[4] = {z0.x, z0.y, z0.z, z0.w};
  float uu[4] = {0.f, 0.f, 0.f, 0.f};
  if (pair) {
    const float4 u = sum_block(rb + 1);
    uu[0] = u.x; uu[1] = u.y; uu[2] = u.z; uu[3] = u.w;
  }
  sk_emit(p, rb, tb, g, lane, v, uu);
}

// The whole product in one launch, where it has enough 32-row blocks to fill the machine
// without cutting the reduction across workgroups: a workgroup of NW wavefronts owns RB
// adjacent row blocks (RB = 2: a (gate, up) pair, or two blocks that share the activation
// blocks) over the whole reduction, the wavefronts take an NW-th each with the same two-deep
// register prefetch as skinny_stream_kernel, add their accumulators through LDS in a fixed
// order, and wavefront g < 4 applies the activation to accumulator registers 4 g .. and stores.
// DUAL: the odd block of the pair reads the second left operand.
struct SkinnyFusedArgs {
  SkinnyArgs s;
  SkinnyReduceArgs e;
};

template <bool A_TILED, int RB, int NW, bool DUAL>
__global__ void __launch_bounds__(NW * 64) skinny_fused_kernel(const SkinnyFusedArgs q) {
  // blocks per register group: four keep the kernel at three workgroups per CU (at most 168
  // registers per lane); eight, two per CU, measured 4 us slower per step at the OPT-13B shape
  constexpr int U = 4;
  constexpr int NA = DUAL ? 2 : 1;
  extern __shared__ float red_mem[];
  float (*red)[RB][16][64] = (float (*)[RB][16][64])red_mem;   // [NW][RB][16][64]
  const SkinnyArgs& p = q.s;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rb0 = blockIdx.x * RB;
  const int kb_total = (p.K + 15) / 16;
  const int per = (kb_total + NW - 1) / NW;
  const int kb0 = wave * per;
  const int kb1 = min(kb_total, kb0 + per);      // may be empty: the wavefront then adds zeros
  const int kb_last = kb_total - 1;

  const char* wbase[RB];
#pragma unroll
  for (int i = 0; i < RB; ++i) wbase[i] = (const char*)p.Bt + ((int64_t)(rb0 + i) * (p.ldb / 16) * 64 + lane) * 16;
  const char* abase[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    abase[i] = (const char*)(i ? p.A1 : p.A);
    if (A_TILED) abase[i] += (int64_t)lane * 16;
    else abase[i] += ((int64_t)min(lane & 31, p.M - 1) * p.lda + (lane >> 5) * 8) * 2;
  }
  auto wload = [&](int i, int kb) { return *(const u32x4_t*)(wbase[i] + (int64_t)min(kb, kb_last) * 1024); };
  auto aload = [&](int i, int kb) {
    const int k = min(kb, kb_last);
    if (A_TILED) return *(const u32x4_t*)(abase[i] + (int64_t)k * 1024);
    const int col = k * 16 + (lane >> 5) * 8;     // a chunk past K reads the row's first chunk (weights are zero there)
    return *(const u32x4_t*)(abase[i] + (col < p.K ? (int64_t)k * 32 : -(int64_t)((lane >> 5) * 16)));
  };
  f32x16_t acc[RB];
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  u32x4_t w0[RB][U], a0[NA][U], w1[RB][U], a1[NA][U];
  auto load = [&](u32x4_t (*w)[U], u32x4_t (*a)[U], int kb) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int i = 0; i < RB; ++i) w[i][u] = wload(i, kb + u);
#pragma unroll
      for (int i = 0; i < NA; ++i) a[i][u] = aload(i, kb + u);
    }
  };
  auto compute = [&](u32x4_t (*w)[U], u32x4_t (*a)[U], int kb) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        SFrag wf, af;
        wf.u = w[i][u];
        af.u = (kb + u < kb1) ? a[DUAL ? i : 0][u] : u32x4_t{0, 0, 0, 0};
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf.v, af.v, acc[i], 0, 0, 0);
      }
  };
  load(w0, a0, kb0);
  for (int kb = kb0; kb < kb1; kb += 2 * U) {
    // (the scheduling barriers keep each batch of loads ahead of the arithmetic of the batch before)
    load(w1, a1, kb + U);
    __builtin_amdgcn_sched_barrier(0);
    compute(w0, a0, kb);
    __builtin_amdgcn_sched_barrier(0);
    load(w0, a0, kb + 2 * U);
    __builtin_amdgcn_sched_barrier(0);
    compute(w1, a1, kb + U);
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave][i][v][lane] = acc[i][v];
  __syncthreads();
  if (wave >= 4) return;
  const int g = wave;
  float sum[RB][4];
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float t = red[0][i][4 * g + e][lane];
      for (int w = 1; w < NW; ++w) t += red[w][i][4 * g + e][lane];
      sum[i][e] = t;
    }
  const bool pair = q.e.act == ACT_GLU && rb0 * 32 < q.e.act_cols;
  if (RB == 2 && pair) {
    sk_emit(q.e, rb0, 0, g, lane, sum[0], sum[RB - 1]);
  } else {
    const float none[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < RB; ++i) sk_emit(q.e, rb0 + i, 0, g, lane, sum[i], none);
  }
}

}  // namespace

int skinny_token_blocks(int M) { return M <= 32 ? 1 : 2; }

size_t skinny_part_bytes(int n_max, int M) {
  // at most ~2048 wavefront tasks: n_rb * n_split <= 2048 + n_rb, one 4 KiB tile each per block of 32 tokens
  return (size_t)(2048 + (n_max + 31) / 32) * 4096 * skinny_token_blocks(M);
}

// g as for the large-batch launcher (M <= 32; destinations tiled with one row block, or
// row-major); part: scratch of skinny_part_bytes(N) bytes.
static void fill_reduce_args(SkinnyReduceArgs& r, const GemmArgs& g, int act) {
  r.n_rb = g.N / 32; r.M = g.M; r.N = g.N;
  r.act = act; r.act_cols = g.act_cols; r.split_col = g.split_col;
  r.C0 = g.C0; r.C1 = g.C1; r.ldc0 = g.ldc0; r.ldc1 = g.ldc1;
  r.c0_tiled = g.c0_tiled; r.c1_tiled = g.c1_tiled; r.n_store = g.n_store;
  r.bias = g.bias; r.bias_cols = g.bias_cols; r.resid = g.resid; r.ldr = g.ldr; r.out_f32 = g.out_f32;
}

template <bool AT, int RB, int NW, bool DUAL>
static int launch_fused_cfg(const SkinnyFusedArgs& q, hipStream_t st) {
  hipLaunchKernelGGL((skinny_fused_kernel<AT, RB, NW, DUAL>), dim3(q.s.n_rb / RB), dim3(NW * 64), (size_t)NW * RB * 4096,
                     st, q);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// 0 launched, -1 failed, 1 not applicable (too few row blocks for one workgroup per RB of them,
// or a reduction too short to share among the wavefronts)
static int launch_skinny_fused(const SkinnyArgs& a, const GemmArgs& g, int act, int kb_total, hipStream_t st) {
  SkinnyFusedArgs q = {};
  q.s = a;
  fill_reduce_args(q.e, g, act);
  q.e.n_tb = 1; q.e.nt = 1;
  const bool at = g.a_tiled != 0, dual = g.A1 != nullptr, glu = act == ACT_GLU;
  const int n_rb = a.n_rb;
  if (dual) {
    if (!at || !glu || (n_rb & 1) || n_rb / 2 < 256 || kb_total < 4 * 4) return 1;
    return launch_fused_cfg<true, 2, 4, true>(q, st);
  }
  if (!(n_rb & 1) && n_rb / 2 >= 256 && kb_total >= 4 * 8)
    return at ? launch_fused_cfg<true, 2, 4, false>(q, st) : launch_fused_cfg<false, 2, 4, false>(q, st);
  // Fewer than about a hundred workgroups cannot pull the weights fast enough (measured: 40-66
  // workgroups of 8-16 wavefronts took 1.4-2x the time of the split version with its reduce).
  if (glu) {   // (gate, up) pairs stay in one workgroup
    if (!(n_rb & 1) && n_rb / 2 >= 96 && kb_total >= 8 * 8)
      return at ? launch_fused_cfg<true, 2, 8, false>(q, st) : launch_fused_cfg<false, 2, 8, false>(q, st);
    return 1;
  }
  if (n_rb >= 96 && kb_total >= 8 * 8)
    return at ? launch_fused_cfg<true, 1, 8, false>(q, st) : launch_fused_cfg<false, 1, 8, false>(q, st);
  return 1;
}

int launch_skinny_bf16(const GemmArgs& g, int act, float* part, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0) return 0;
  if (g.M > SKINNY_MAX_M || (g.N & 31) || g.partial) return -1;
  const int nt = skinny_token_blocks(g.M);
  SkinnyArgs a = {};
  a.n_tb = (g.M + 31) / 32;
  a.A = g.A; a.A1 = g.A1; a.Bt = g.Bt; a.lda = g.lda; a.ldb = g.ldb;
  a.M = g.M; a.N = g.N; a.K = g.K; a.a_tiled = g.a_tiled;
  a.n_rb = g.N / 32;
  const int kb_total = (g.K + 15) / 16;
  if (nt == 1) {
    const int fused = launch_skinny_fused(a, g, act, kb_total, st);
    if (fused <= 0) return fused;   // launched (0) or failed (-1); 1 = not applicable
  }
  // enough ranges for about 1024 wavefronts (one per SIMD), at least 32 blocks (32 KiB of weights)
  // each.  Measured per decode step (Llama shape / OPT-13B shape): 2048 wavefronts 48.5 / 60.8 us,
  // 1024: 48.4 / 56.6, 768: 49.5 / 56.9, 512: 50.8 / 60.4; 16 blocks each: 53.1 / 62.0, 64: 52.7 / 59.7.
  const int max_s = kb_total / 32 > 0 ? kb_total / 32 : 1;
  int S = 1024 / a.n_rb;
  if (S > max_s) S = max_s;
  if (S < 1) S = 1;
  a.kb_per = (kb_total + S - 1) / S;
  a.n_split = (kb_total + a.kb_per - 1) / a.kb_per;
  a.part = part;
  const int tasks = a.n_rb * a.n_split;
  const dim3 grid((tasks + 3) / 4), blk(256);
  if (g.a_tiled) {
    if (nt == 1) hipLaunchKernelGGL((skinny_stream_kernel<true, 1>), grid, blk, 0, st, a);
    else hipLaunchKernelGGL((skinny_stream_kernel<true, 2>), grid, blk, 0, st, a);
  } else {
    if (nt == 1) hipLaunchKernelGGL((skinny_stream_kernel<false, 1>), grid, blk, 0, st, a);
    else hipLaunchKernelGGL((skinny_stream_kernel<false, 2>), grid, blk, 0, st, a);
  }
  if (hipGetLastError() != hipSuccess) return -1;
  SkinnyReduceArgs r = {};
  fill_reduce_args(r, g, act);
  r.part = part; r.n_split = a.n_split; r.rb_split = r.n_rb; r.n_split_b = a.n_split;
  r.n_tb = a.n_tb; r.nt = nt;
  hipLaunchKernelGGL(skinny_reduce_kernel, dim3(r.n_rb * r.n_tb), dim3(256), 0, st, r);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_skinny_reduce(const GemmArgs& g, int act, const float* part, int n_split, int f16_out, hipStream_t st) {
  return launch_skinny_reduce2(g, act, part, n_split, g.N / 32, n_split, f16_out, st);
}

int launch_skinny_reduce2(const GemmArgs& g, int act, const float* part, int n_split, int rb_split, int n_split_b,
                          int f16_out, hipStream_t st) {
  SkinnyReduceArgs r = {};
  r.f16_out = f16_out; r.rb_split = rb_split; r.n_split_b = n_split_b; r.n_tb = 1; r.nt = 1;
  r.part = part; r.n_rb = g.N / 32; r.n_split = n_split; r.M = g.M; r.N = g.N;
  r.act = act; r.act_cols = g.act_cols; r.split_col = g.split_col;
  r.C0 = g.C0; r.C1 = g.C1; r.ldc0 = g.ldc0; r.ldc1 = g.ldc1;
  r.c0_tiled = g.c0_tiled; r.c1_tiled = g.c1_tiled; r.n_store = g.n_store;
  r.bias = g.bias; r.bias_cols = g.bias_cols; r.resid = g.resid; r.ldr = g.ldr; r.out_f32 = g.out_f32;
  hipLaunchKernelGGL(skinny_reduce_kernel, dim3(r.n_rb), dim3(256), 0, st, r);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

constexpr int SKQ_MAX_SPLIT = 32;
size_t skinny_q_part_bytes(int n_max) {
  // two streamed segments per product, each at most SKQ_MAX_SPLIT ranges of one 4 KiB tile per row block
  return (size_t)2 * SKQ_MAX_SPLIT * ((n_max + 31) / 32) * 4096;
}

// kernel arguments and workgroup count of one part (0 workgroups if it is empty)
static int q_part_args(const GemmArgs& g, const SkinnyQ& q, float* part, int slot0, int rb_out0, int n_rb_part,
                       int max_wgs, SkinnyQArgs* out, int* wgs) {
  *wgs = 0;
  SkinnyQArgs a = {};
  *out = a;
  if (g.N <= 0 || g.K <= 0) return 0;
  if (g.M <= 0 || g.M > 32 || (g.K & 63) || (q.bits != 3 && q.bits != 8)) return -1;
  if ((q.down != 0) != (g.a_tiled != 0) || (!q.down && (g.K & 127))) return -1;
  const int rbs = skq_rb(q.bits, q.down != 0);
  if (g.N % (32 * rbs)) return -1;
  a.A = g.A; a.lda = g.lda; a.M = g.M;
  a.n_rb = g.N / 32;
  const int n_rbg = a.n_rb / rbs;
  const int ub = q.down ? 1 : 2;
  a.nu_total = g.K / (64 * ub);
  // ranges: about 512 workgroups, at least two units per wavefront, and partial tiles (4 KiB
  // per row block and range) of at most half of the packed weights' bytes
  const size_t wbytes = (size_t)a.n_rb * (g.K / 64) * qblock_bytes(q.bits);
  int S = (512 + n_rbg - 1) / n_rbg;
  if (S > a.nu_total / 8) S = a.nu_total / 8;
  const int cap = (int)(wbytes / ((size_t)8192 * a.n_rb));
  if (S > cap) S = cap;
  if (S > SKQ_MAX_SPLIT) S = SKQ_MAX_SPLIT;
  if (S > max_wgs / n_rbg) S = max_wgs / n_rbg;
  if (S < 1) S = 1;
  a.nu_per = (a.nu_total + S - 1) / S;
  a.n_split = (a.nu_total + a.nu_per - 1) / a.nu_per;
  a.slot0 = slot0; a.rb_out0 = rb_out0; a.n_rb_part = n_rb_part;
  a.codes = (const char*)q.codes; a.scales = (const uint16_t*)q.scales; a.G = q.G; a.Kp = q.Kp;
  a.part = part;
  *out = a;
  *wgs = n_rbg * a.n_split;
  return 0;
}

int launch_skinny_q_pair(const GemmArgs& g8, const SkinnyQ& q8, const GemmArgs& g3, const SkinnyQ& q3, float* part,
                         int n_split[2], hipStream_t st) {
  n_split[0] = n_split[1] = 0;
  const bool down = (g8.N > 0 && g8.K > 0) ? q8.down != 0 : q3.down != 0;
  SkinnyQ2Args a = {};
  int w8 = 0, w3 = 0;
  // The kernels hold three workgroups per CU: the 3-bit part takes its ranges first, the 8-bit
  // part what is left of one full round (768 workgroups), so that no second round starts for a
  // few workgroups.
  constexpr int ROUND = 768;
  if (down) {
    // same rows, two segments of the reduction: the 3-bit ranges follow the 8-bit ones
    const int n_rb = (g8.N > 0 ? g8.N : g3.N) / 32;
    if (q_part_args(g3, q3, part, 0, 0, n_rb, ROUND, &a.s3, &w3)) return -1;
    if (q_part_args(g8, q8, part, 0, 0, n_rb, ROUND - w3, &a.s8, &w8)) return -1;
    a.s3.slot0 = a.s8.n_split;
  } else {
    // two row ranges of one output: the 3-bit rows follow the 8-bit rows
    const int n_rb = (g8.N > 0 ? g8.N / 32 : 0) + (g3.N > 0 ? g3.N / 32 : 0);
    if (q_part_args(g3, q3, part, 0, g8.N > 0 ? g8.N / 32 : 0, n_rb, ROUND, &a.s3, &w3)) return -1;
    if (q_part_args(g8, q8, part, 0, 0, n_rb, ROUND - w3, &a.s8, &w8)) return -1;
  }
  if (w8 + w3 == 0) return 0;
  a.wg8 = w8;
  // LDS: the four wavefronts' accumulators of the row blocks, [4][RB][16][64] floats
  constexpr int rb_dn = skq_rb(3, true) > skq_rb(8, true) ? skq_rb(3, true) : skq_rb(8, true);
  constexpr int rb_up = skq_rb(3, false) > skq_rb(8, false) ? skq_rb(3, false) : skq_rb(8, false);
  if (down) hipLaunchKernelGGL(skinny_stream_q2_kernel<true>, dim3(w8 + w3), dim3(256), 4 * rb_dn * 4096, st, a);
  else hipLaunchKernelGGL(skinny_stream_q2_kernel<false>, dim3(w8 + w3), dim3(256), 4 * rb_up * 4096, st, a);
  if (hipGetLastError() != hipSuccess) return -1;
  n_split[0] = a.s8.n_split; n_split[1] = a.s3.n_split;
  return 0;
}

}  // namespace ffsplit
