// The low-rank remainder's two middle products in one kernel (Eq. 2, FFN_2 with the factors of
// Sec. 4.2 / 5.1.1):   t2 = gelu(t * Q1) * P2   without storing h2 = gelu(t * Q1).
//
// A workgroup owns 128 token rows and a range of neurons.  It walks its neurons in chunks of
// 256: phase 1 computes the chunk's pre-activations [128, 256] from the tile of t (reduction
// over the rank, 512), applies GeLU and parks the result as bf16 in LDS in the operand layout of
// the MFMA; phase 2 multiplies that by the chunk's 256 rows of P2 into the workgroup's
// [128, 512] fp32 accumulators, which live in registers for the whole walk.  The neuron ranges
// of one row tile are summed afterwards in a fixed order (fp32 partials, the same format as
// the split-K partials of the separate h2 * P2 product).  Rank 512 only: the accumulators of a
// larger rank do not fit the register file at a row count that feeds the matrix cores.
//
// All operands are in the tiled layout (32 rows x 16 reduction elements per 1 KiB block, see
// gemm_bf16.hip) and go from global memory straight into a ring of LDS stages; one slab is 32
// rank elements of (t tile, Q1 chunk) in phase 1 and 16 neurons of the P2 chunk in phase 2, so
// the ring keeps running across the phases and across chunks.
#include "common.h"
#include <atomic>
#include <type_traits>
#include <utility>

namespace ffsplit {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

union Frag {
  u32x4_t u;
  bf16x8_t v;
};

constexpr int FBM = 128;                   // token rows of a workgroup
constexpr int FC = 256;                    // neurons per chunk
constexpr int FR = 512;                    // rank (padded) = columns of t and of t2
constexpr int NWAVE = 4;                   // 2 (rows) x 2 (columns), one per SIMD: 512 registers per lane
constexpr int STAGES = 4;
constexpr int STAGE_BLK = 24;              // 1 KiB blocks per stage
constexpr int P1_SLABS = FR / 32;          // phase 1: 32 rank elements per slab (8 + 16 blocks)
constexpr int P2_SLABS = FC / 16;          // phase 2: 16 neurons per slab (16 blocks)
constexpr int SLABS = P1_SLABS + P2_SLABS; // per chunk; a multiple of STAGES: static stage per position
constexpr int STEPS = 2 * P1_SLABS + P2_SLABS;   // k steps of 16 per chunk
constexpr int H2_BLK = (FBM / 32) * (FC / 16);   // the parked chunk: 64 blocks
constexpr size_t LDS_BYTES = (size_t)(STAGES * STAGE_BLK + H2_BLK) * 1024;
static_assert(SLABS % STAGES == 0, "stage of a slab position must not depend on the chunk");
static_assert(LDS_BYTES <= 160 * 1024, "LDS of a CU");

struct Ffn2Args {
  const char* T1;    // t, tiled [rows / 32][FR / 16] blocks
  const char* Q1t;   // tiled [mp / 32][FR / 16]
  const char* P2t;   // tiled [FR / 32][mp / 16]
  float* part;       // [n_split][M][FR]
  int M, mp;
  int row_tiles, n_split;
  int chunks, chunks_per_split;
};

__device__ __forceinline__ int xcd_remap(int i, int total) {
  const int q = total >> 3, rem = total & 7, x = i & 7;
  return x * q + (x < rem ? x : rem) + (i >> 3);
}
__device__ __forceinline__ void swap32(uint32_t& a, uint32_t& b) {
  auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  a = r[0];
  b = r[1];
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}
template <int... I, class F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}

// loads per wavefront of the slab at position p of a chunk (positions past the chunk belong to
// the next one, which exists unless LAST)
template <bool LAST>
constexpr int loads_of(int p) {
  if (p >= SLABS) return LAST ? 0 : loads_of<false>(p - SLABS);
  return p < P1_SLABS ? 6 : 4;
}
// slab of k step s of a chunk, and whether s is the last step of its slab
constexpr int slab_of(int s) { return s < 2 * P1_SLABS ? s / 2 : P1_SLABS + (s - 2 * P1_SLABS); }
constexpr bool last_of_slab(int s) { return s < 2 * P1_SLABS ? (s & 1) == 1 : true; }

__global__ void __launch_bounds__(NWAVE * 64) __attribute__((amdgpu_waves_per_eu(1, 1)))
ffn2_fused_kernel(const Ffn2Args p) {
  extern __shared__ u32x4_t smem[];
  u32x4_t* const h2c = smem + STAGES * STAGE_BLK * 64;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int logical = xcd_remap(blockIdx.x, p.row_tiles * p.n_split);
  // (consecutive logical indices share an XCD and its L2: the workgroups of one neuron range,
  // which stream the same weights)
  const int split = logical / p.row_tiles, tm = logical % p.row_tiles;
  const int m0 = tm * FBM;
  const int c_first = split * p.chunks_per_split;
  const int c_end = min(p.chunks, c_first + p.chunks_per_split);   // >= c_first + 1 by the host's choice

  // ---- sources.  Phase 1, wavefront w: blocks w, w + 4 of the t tile (row block idx / 2, k block
  // idx % 2) and blocks w, w + 4, w + 8, w + 12 of the Q1 chunk (likewise).  Phase 2: rows w,
  // w + 4, w + 8, w + 12 of the 16 row blocks of P2.  Row blocks past the matrices repeat the last one; the
  // neurons concerned are zeroed after the activation.
  const int t_rb_last = (p.M + 31) / 32 - 1, q_rb_last = p.mp / 32 - 1, p2_kb_last = p.mp / 16 - 1;
  const int p2_ldb = p.mp / 16;   // k blocks per row block of P2t
  const char* t_src[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = wave + 4 * i;
    int grb = m0 / 32 + (idx >> 1);
    grb = grb <= t_rb_last ? grb : t_rb_last;
    t_src[i] = p.T1 + ((int64_t)grb * (FR / 16) + (idx & 1)) * 1024;
  }
  // (every source address is a wavefront-uniform block address plus the lane's 16 bytes: the
  // block addresses stay in scalar registers)
  const uint32_t lane16 = lane * 16;
  auto dma = [&](const char* blk, u32x4_t* dst) __attribute__((always_inline)) {
    uint64_t b = (uint64_t)blk;
    asm("" : "+s"(b));   // (keeps the block address a scalar pair: not folded into a per-lane pointer)
    __builtin_amdgcn_global_load_lds((gptr_t)((const char*)b + lane16), (lptr_t)dst, 16, 0, 0);
  };
  // the loads of the slab at position pos (static) of chunk gc
  auto issue = [&](int gc, auto posc) __attribute__((always_inline)) {
    constexpr int pos = decltype(posc)::value;
    u32x4_t* st = smem + (pos % STAGES) * (STAGE_BLK * 64);
    if constexpr (pos < P1_SLABS) {
#pragma unroll
      for (int i = 0; i < 2; ++i) dma(t_src[i] + pos * 2048, st + (wave + 4 * i) * 64);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int idx = wave + 4 * i;
        int rb = gc * (FC / 32) + (idx >> 1);
        rb = rb <= q_rb_last ? rb : q_rb_last;
        dma(p.Q1t + ((int64_t)rb * (FR / 16) + 2 * pos + (idx & 1)) * 1024, st + (8 + idx) * 64);
      }
    } else {
      int kb = gc * (FC / 16) + (pos - P1_SLABS);
      kb = kb <= p2_kb_last ? kb : p2_kb_last;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rb = wave + 4 * i;
        dma(p.P2t + ((int64_t)rb * p2_ldb + kb) * 1024, st + rb * 64);
      }
    }
  };

  f32x16_t acc2[2][8];   // t2 tile: rows wm * 64 + 32 i, columns wn * 256 + 32 j
  f32x16_t acc1[2][4];   // chunk pre-activations: rows wm * 64 + 32 i, neurons wn * 128 + 32 j
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc2[i][j][v] = 0.f;

  // Fragment registers of two consecutive k steps.
  Frag fa[2][2], fb[2][8];
  // the lane's LDS bases: every access is one of these plus a compile-time offset
  const u32x4_t* const ringA = smem + (wm * 2 * 2) * 64 + lane;        // phase 1, t tile
  const u32x4_t* const ringB1 = smem + (8 + wn * 4 * 2) * 64 + lane;   // phase 1, Q1 chunk
  const u32x4_t* const ringB2 = smem + (wn * 8) * 64 + lane;           // phase 2, P2 chunk
  u32x4_t* const h2w = h2c + ((wm * 2) * (FC / 16) + wn * 8) * 64 + lane;   // parked chunk, this wavefront's part
  const u32x4_t* const h2r = h2c + ((wm * 2) * (FC / 16)) * 64 + lane;      // ... its row blocks
  // the weights' fragments of step s (from the ring) / the tokens' fragments (ring in phase 1,
  // the parked chunk in phase 2)
  auto read_b = [&](auto sc) __attribute__((always_inline)) {
    constexpr int s = decltype(sc)::value, set = s & 1, pos = slab_of(s);
    constexpr int st = (pos % STAGES) * (STAGE_BLK * 64);
    if constexpr (pos < P1_SLABS) {
      constexpr int ks = s & 1;
#pragma unroll
      for (int j = 0; j < 4; ++j) fb[set][j].u = ringB1[st + (j * 2 + ks) * 64];
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) fb[set][j].u = ringB2[st + j * 64];
    }
  };
  auto read_a = [&](auto sc) __attribute__((always_inline)) {
    constexpr int s = decltype(sc)::value, set = s & 1, pos = slab_of(s);
    if constexpr (pos < P1_SLABS) {
      constexpr int ks = s & 1;
      constexpr int st = (pos % STAGES) * (STAGE_BLK * 64);
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[set][i].u = ringA[st + (i * 2 + ks) * 64];
    } else {
      constexpr int kb = pos - P1_SLABS;
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[set][i].u = h2r[(i * (FC / 16) + kb) * 64];
    }
  };
  // (weights as the first operand: a lane then holds four consecutive columns of one row)
  auto mfma = [&](auto sc) __attribute__((always_inline)) {
    constexpr int s = decltype(sc)::value, set = s & 1;
    if constexpr (slab_of(s) < P1_SLABS) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc1[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j].v, fa[set][i].v, acc1[i][j], 0, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
          acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j].v, fa[set][i].v, acc2[i][j], 0, 0, 0);
    }
  };
  // GeLU of the chunk's pre-activations -> bf16 -> the parked chunk, tiled: block (row block,
  // 16 neurons), lane = 32 (neuron / 8 % 2) + row
  auto park = [&](int gc) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool live = gc * FC + wn * 128 + j * 32 < p.mp;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        uint32_t pk[4][2];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = live ? gelu_fast(acc1[i][j][4 * g + e]) : 0.f;
          pk[g][0] = pack_bf16x2(v[0], v[1]);
          pk[g][1] = pack_bf16x2(v[2], v[3]);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          swap32(pk[2 * t][0], pk[2 * t + 1][0]);
          swap32(pk[2 * t][1], pk[2 * t + 1][1]);
          const u32x4_t val = {pk[2 * t][0], pk[2 * t][1], pk[2 * t + 1][0], pk[2 * t + 1][1]};
          h2w[(i * (FC / 16) + j * 2 + t) * 64] = val;
        }
      }
    }
  };
  // The barrier that publishes the slab at position pos (its loads have landed in every wavefront)
  // and retires the one before it (every wavefront's reads of it are complete).  At that point
  // the loads of the two following slabs may still be in flight.
  auto publish = [&](auto posc, auto lastc) __attribute__((always_inline)) {
    constexpr int pos = decltype(posc)::value;
    constexpr bool LAST = decltype(lastc)::value;
    wait_vmcnt<loads_of<LAST>(pos + 1) + loads_of<LAST>(pos + 2)>();
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  };

  // One chunk: its 48 k steps.  On entry the fragments of step 0 are in set 0, slabs 0 is
  // published, and the loads up to slab 3 are issued.  During step s the fragments of step s + 1
  // are read; once those reads are the last of their slab, the barrier of the next slab follows
  // and the stage just retired is refilled four slabs ahead.
  auto chunk = [&](int gc, auto lastc) __attribute__((always_inline)) {
    constexpr bool LAST = decltype(lastc)::value;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc1[i][j][v] = 0.f;
    static_for(std::make_integer_sequence<int, STEPS>{}, [&](auto sc) __attribute__((always_inline)) {
      constexpr int s = decltype(sc)::value;
      constexpr int n = s + 1;                     // the step read ahead
      constexpr bool have_next = n < STEPS || !LAST;
      constexpr int ns = n % STEPS;                // ... as a step of its own chunk
      constexpr bool park_here = (n == 2 * P1_SLABS);   // step n needs the parked chunk
      // the slab retired by the barrier that preceded this step is refilled now: that barrier
      // was publish(q) with q = slab_of(s) + 1 when step s is the last of its slab
      if constexpr (have_next) {
        read_b(std::integral_constant<int, ns>{});
        if constexpr (!park_here) read_a(std::integral_constant<int, ns>{});
      }
      if constexpr (last_of_slab(s)) {
        constexpr int fill = slab_of(s) + STAGES;   // = (slab_of(s) + 1) + STAGES - 1
        if constexpr (fill < SLABS) issue(gc, std::integral_constant<int, fill>{});
        else if constexpr (!LAST) issue(gc + 1, std::integral_constant<int, fill - SLABS>{});
      }
      mfma(sc);
      {
        // Instruction order of the step: the LDS reads of the next step, then the direct loads,
        // dealt out evenly between the MFMAs (bursts of memory instructions stall the issuing
        // wavefront and with it the matrix pipeline)
        constexpr int NM = slab_of(s) < P1_SLABS ? 8 : 16;
        constexpr int NR = !have_next ? 0 : (slab_of(ns) < P1_SLABS ? 6 : (park_here ? 8 : 10));
        constexpr int fillp = slab_of(s) + STAGES;
        constexpr int NL = !last_of_slab(s) ? 0 : loads_of<LAST>(fillp);
        constexpr int TOT = NR + NL, PER = TOT / NM, REM = TOT % NM;
        int done = 0;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          const int cnt = PER + (m < REM ? 1 : 0);
#pragma unroll
          for (int q = 0; q < cnt; ++q) {
            if (done < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            else __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
            ++done;
          }
        }
      }
      if constexpr (park_here) park(gc);
      if constexpr (have_next && last_of_slab(ns)) {
        // step n is the last of its slab: the barrier of the slab after it
        constexpr int q = slab_of(ns) + 1 + (n >= STEPS ? SLABS : 0);
        if constexpr (q < SLABS || !LAST) publish(std::integral_constant<int, q>{}, lastc);
      }
      if constexpr (park_here) read_a(std::integral_constant<int, ns>{});
    });
  };

  // prologue: slabs 0 .. 2 of the first chunk, its barrier, slab 3, the first fragments
  issue(c_first, std::integral_constant<int, 0>{});
  issue(c_first, std::integral_constant<int, 1>{});
  issue(c_first, std::integral_constant<int, 2>{});
  wait_vmcnt<loads_of<false>(1) + loads_of<false>(2)>();
  asm volatile("s_barrier" ::: "memory");
  issue(c_first, std::integral_constant<int, 3>{});
  read_b(std::integral_constant<int, 0>{});
  read_a(std::integral_constant<int, 0>{});

#pragma unroll 1
  for (int gc = c_first; gc < c_end - 1; ++gc) chunk(gc, std::false_type{});
  chunk(c_end - 1, std::true_type{});

  // ---- fp32 partials [split][M][FR]: lane: row lane & 31, columns 8 g + 4 (lane >> 5) + 0..3
  const int half = lane >> 5;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = m0 + wm * 64 + i * 32 + (lane & 31);
    if (row >= p.M) continue;
    float* dst = p.part + ((int64_t)split * p.M + row) * FR + wn * 256 + 4 * half;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *(float4*)(dst + j * 32 + 8 * g) = make_float4(acc2[i][j][4 * g], acc2[i][j][4 * g + 1], acc2[i][j][4 * g + 2],
                                                       acc2[i][j][4 * g + 3]);
  }
}

}  // namespace

int ffn2_fused_splits(int M, int mp) {
  if (M <= 0 || mp <= 0) return 0;
  const int row_tiles = (M + FBM - 1) / FBM, chunks = (mp + FC - 1) / FC;
  int S = 256 / row_tiles;
  if (S < 1) S = 1;
  if (S > chunks) S = chunks;
  const int cps = (chunks + S - 1) / S;
  return (chunks + cps - 1) / cps;
}

int launch_ffn2_fused(const void* T1, int64_t ldt, const void* Q1t, int64_t ldq, const void* P2t, int64_t ldp2, int M,
                      int mp, int rp, float* part, int n_split, hipStream_t st) {
  if (!T1 || !Q1t || !P2t || !part) return -1;
  if (rp != FR || ldt != FR || ldq != FR || ldp2 != mp || mp < 64 || (mp & 63) || M <= 0) return -1;
  if (n_split != ffn2_fused_splits(M, mp)) return -1;
  Ffn2Args a = {};
  a.T1 = (const char*)T1; a.Q1t = (const char*)Q1t; a.P2t = (const char*)P2t; a.part = part;
  a.M = M; a.mp = mp;
  a.row_tiles = (M + FBM - 1) / FBM;
  a.n_split = n_split;
  a.chunks = (mp + FC - 1) / FC;
  a.chunks_per_split = (a.chunks + n_split - 1) / n_split;
  if ((int64_t)(n_split - 1) * a.chunks_per_split >= a.chunks) return -1;   // every split has a chunk
  // more dynamic LDS than the default limit: set once per device (a set-once bit mask per device
  // ordinal is the only state; racing first calls set it twice, harmlessly).  A device that
  // refuses the size is reported as unsupported (1) and stays so.
  static std::atomic<uint64_t> configured{0}, refused{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return -1;
  const uint64_t bit = 1ull << (dev & 63);
  if (dev < 64 && (refused.load(std::memory_order_acquire) & bit)) return 1;
  if (dev >= 64 || !(configured.load(std::memory_order_acquire) & bit)) {
    if (hipFuncSetAttribute((const void*)ffn2_fused_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)LDS_BYTES) != hipSuccess) {
      (void)hipGetLastError();
      if (dev < 64) refused.fetch_or(bit, std::memory_order_release);
      return 1;
    }
    if (dev < 64) configured.fetch_or(bit, std::memory_order_release);
  }
  hipLaunchKernelGGL(ffn2_fused_kernel, dim3(a.row_tiles * n_split), dim3(NWAVE * 64), LDS_BYTES, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace ffsplit
