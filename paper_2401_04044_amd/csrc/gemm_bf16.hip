// bf16 MFMA GEMM of the split feed-forward path, gfx950 only.
//
//   D[M, N] = A[M, K] * B[N, K]^T ,  fp32 accumulation, fused epilogue.
//
// Data layouts
//   "tiled": the matrix is cut into blocks of 32 rows x 16 k-elements (1 KiB).
//     Inside a block the 16-byte chunk of lane l = 32 c + r holds row r,
//     k-elements 8 c .. 8 c + 7, which is exactly the operand register image of
//     v_mfma_f32_32x32x16_bf16.  Blocks are ordered [row block][k block], so a
//     K slab of one row block is contiguous.  All packed weights and all
//     intermediates between the chained products use this layout: global loads
//     and LDS reads are then contiguous 1 KiB per wavefront instruction and free
//     of bank conflicts by construction.
//   "row-major": ordinary [rows, ld] (the caller's X and Y).
//
// Kernel: BM x BN workgroup tile; BK-deep slabs go from global memory straight into a ring of
// LDS stages (global_load_lds_dwordx4, one 1 KiB operand block per wavefront instruction);
// each wavefront owns a (BM/WGM) x (BN/WGN) sub-tile of 32x32 MFMA tiles.  The MFMA is issued
// with the weights as the first operand so that a lane ends up with 4 consecutive output
// columns of one row; one v_permlane32_swap turns that into 8 consecutive columns = one
// 16-byte chunk of the tiled (or row-major) output.
//
// Epilogues: plain / GeLU / SwiGLU (on (gate, up) pairs of 32-column blocks)
// with two output destinations, fp32 split-K partials, and the neuron-norm
// column reduction of Sec. 4.1 (Eq. 3) for the calibration pass.
#include "common.h"
#include <atomic>
#include <type_traits>

namespace ffsplit {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;  // native vector: stays in registers

union Frag {
  u32x4_t u;
  bf16x8_t v;
};

__device__ __forceinline__ int xcd_remap(int i, int total) {
  const int q = total >> 3, rem = total & 7, x = i & 7;
  return x * q + (x < rem ? x : rem) + (i >> 3);
}

template <int ACT>
__device__ __forceinline__ float act_bf16(float z, float g) {
  if (ACT == ACT_GELU) return gelu_fast(z);
  if (ACT == ACT_GLU) return silu_fast(g) * z;
  return z;
}

// swap the upper 32 lanes of a with the lower 32 lanes of b
__device__ __forceinline__ void swap32(uint32_t& a, uint32_t& b) {
  auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  a = r[0];
  b = r[1];
}

// Epilogue shared by the GEMM kernels: activation, bf16 packing and the stores (or the
// neuron-norm column sums).  acc[i][j] is the 32x32 tile (i, j) of the wavefront's sub-tile.
// EPI: the optional additions of GemmArgs (bias, residual stream, fp32 destination) are compiled
// in; the plain instantiations carry none of their instructions.
template <int BM, int BN, int WGM, int WGN, int ACT, bool SCORE, bool EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& p, f32x16_t (&acc)[BM / WGM / 32][BN / WGN / 32], int m0,
                                              int n0, int tm, int wm, int wn, int lane, int tid, u32x4_t* smem) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  // ---------------------------------------------------------------- epilogue
  constexpr int JSTEP = (ACT == ACT_GLU) ? 2 : 1;
  if (!SCORE) {
    // lane: row = lane & 31; columns 8 g + 4 (lane >> 5) + 0..3 of each 32x32 tile
    const int half = lane >> 5;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int cb = n0 + wn * WN + j * 32;  // GEMM column of this 32-block
      if (cb >= p.N) continue;
      const bool act_here = cb < p.act_cols;
      int oc;       // output column of the block
      if (ACT == ACT_GLU) {
        if (act_here) {
          if (j & 1) continue;  // the pair is written when its gate block comes up
          oc = cb / 2;
        } else {
          oc = cb - p.act_cols / 2;
        }
      } else {
        oc = cb;
      }
      char* base;
      int64_t ld;
      int occ, tiled;
      const bool to_c0 = oc < p.split_col;
      if (to_c0) { base = (char*)p.C0; ld = p.ldc0; occ = oc; tiled = p.c0_tiled; }
      else { base = (char*)p.C1; ld = p.ldc1; occ = oc - p.split_col; tiled = p.c1_tiled; }
      // a neuron's bias (GEMM column cb + 8 g + 4 half + e), added before the activation
      float bz[4][4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c = cb + 8 * g + 4 * half;
        float4 b4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (EPI && ACT != ACT_GLU && p.bias != nullptr && c + 3 < p.bias_cols) b4 = *(const float4*)(p.bias + c);
        bz[g][0] = b4.x; bz[g][1] = b4.y; bz[g][2] = b4.z; bz[g][3] = b4.w;
      }
      const bool f32o = EPI && p.out_f32 && to_c0 && !tiled;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int rblk = (m0 + wm * WM) / 32 + i;
        const int row = rblk * 32 + (lane & 31);
        if (p.partial) {
          // fp32 split-K partial, row-major [split][M][ld]
          if (row < p.M) {
            float* dst = (float*)base + ((int64_t)blockIdx.y * p.M + row) * ld + occ + 4 * half;
#pragma unroll
            for (int g = 0; g < 4; ++g)
              *(float4*)(dst + 8 * g) = make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                                                    acc[i][j][4 * g + 3]);
          }
          continue;
        }
        // the residual stream (fp32, row-major, same columns as the destination)
        // (un-activated products start their accumulators from the residual instead: see the kernel)
        const float* rrow = (EPI && ACT != ACT_NONE && p.resid != nullptr && to_c0 && !tiled && row < p.M)
                                ? p.resid + (int64_t)row * p.ldr + occ + 4 * half : nullptr;
        uint32_t pk[4][2];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            // (static tile indices: an activated pair is (gate j, value j + 1))
            constexpr int TNM1 = TN - 1;
            const int j1 = j + 1 < TN ? j + 1 : TNM1;
            const float gt = EPI ? acc[i][j][4 * g + e] + bz[g][e] : acc[i][j][4 * g + e];
            const float z = (ACT == ACT_GLU && act_here) ? acc[i][j1][4 * g + e] : gt;
            v[e] = act_here ? act_bf16<ACT>(z, gt) : z;
          }
          const bool col_ok = occ + 8 * g + 4 * half < p.n_store;
          if (EPI && rrow != nullptr && col_ok) {
            const float4 r4 = *(const float4*)(rrow + 8 * g);
            v[0] += r4.x; v[1] += r4.y; v[2] += r4.z; v[3] += r4.w;
          }
          if (EPI && f32o) {
            if (row < p.M && col_ok)
              *(float4*)((float*)base + (int64_t)row * ld + occ + 8 * g + 4 * half) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
            pk[g][0] = pack_bf16x2(v[0], v[1]);
            pk[g][1] = pack_bf16x2(v[2], v[3]);
          }
        }
        if (EPI && f32o) continue;
        // groups (0,1) and (2,3) each cover 16 consecutive columns: after the swap the lower
        // lanes hold columns 0..7 and the upper lanes columns 8..15 of those 16
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          swap32(pk[2 * t][0], pk[2 * t + 1][0]);
          swap32(pk[2 * t][1], pk[2 * t + 1][1]);
          const u32x4_t val = {pk[2 * t][0], pk[2 * t][1], pk[2 * t + 1][0], pk[2 * t + 1][1]};
          const int col = occ + 16 * t;  // block of 16 output columns
          if (tiled) {
            if (rblk * 32 < p.m_pad)
              *(u32x4_t*)(base + (((int64_t)rblk * (ld / 16) + col / 16) * 64 + lane) * 16) = val;
          } else {
            if (row < p.M && col + 8 * half < p.n_store)
              *(u32x4_t*)(base + ((int64_t)row * ld + col + 8 * half) * 2) = val;
          }
        }
      }
    }
  } else {
    // lane: column = lane & 31; rows 8 g + 4 (lane >> 5) + 0..3 of each 32x32 tile
    constexpr int BNO = BN / JSTEP;
    float* red2 = (float*)smem;  // [WGM][BNO]
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
          // same activation forms as the forward epilogue: the scores rank what the forward computes
          // (the erf form costs about a fifth of the calibration pass, nothing hides it at one
          // workgroup per CU)
          float h = act_bf16<ACT>(z, gt);
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

// ---------------------------------------------------------------------------------------------
// Direct-to-LDS variant: every wavefront instruction moves one 1 KiB operand block from global
// memory straight into its LDS slot (global_load_lds_dwordx4), STAGES slabs deep, no staging
// registers and no LDS store instructions.  One barrier per slab: it publishes the slab that is
// about to be consumed and retires the one consumed last, whose slot the new loads overwrite.
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in
// imm[3:0] and imm[15:14], expcnt imm[6:4], lgkmcnt imm[11:8])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}
// workgroup barrier without a memory fence (the kernel orders its loads with explicit counters);
// the memory clobber keeps the compiler from moving LDS accesses across it
__device__ __forceinline__ void lds_barrier() { asm volatile("s_barrier" ::: "memory"); }

// KG > 1 splits the reduction inside the workgroup: KG groups of WGM x WGN wavefronts each take
// every KG-th part of a slab for the same output tile; the groups' accumulators are summed through
// LDS in a fixed order before the epilogue.  This gives small products (few tiles, long K)
// more wavefronts per CU without partial sums in global memory.
// wavefronts per SIMD the kernel is compiled for: a wave tile of 16 or more 32 x 32 accumulator
// tiles (256+ registers) runs alone on its SIMD, with 512 registers per lane
constexpr int gemm_waves_per_simd(int wm, int wn) { return (wm / 32) * (wn / 32) >= 16 ? 1 : 2; }

template <int BM, int BN, int BK, int WGM, int WGN, int KG, int STAGES, int ACT, bool DUAL, bool SCORE, bool A_TILED,
          bool EPI>
__global__ void __launch_bounds__(WGM* WGN* KG * 64)
    __attribute__((amdgpu_waves_per_eu(gemm_waves_per_simd(BM / WGM, BN / WGN), gemm_waves_per_simd(BM / WGM, BN / WGN))))
gemm_bf16_dl_kernel(const GemmArgs p) {
  constexpr int NWT = WGM * WGN;               // wavefronts per k group
  constexpr int NW = NWT * KG;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int NA = DUAL ? 2 : 1;
  constexpr int KB = BK / 16;                  // k blocks per slab
  constexpr int KS = KB / KG;                  // k steps of a slab per wavefront
  constexpr int A_BLK = NA * (BM / 32) * KB;   // 1 KiB blocks of one slab
  constexpr int B_BLK = (BN / 32) * KB;
  // loads per wavefront and slab; where the weights' blocks do not divide over the wavefronts the
  // last round is padded with repeats of the tile's last row block, which land in spare slots
  // that nothing reads (every wavefront then issues the same number of loads, which the
  // wait counts below rely on)
  constexpr int LA = A_BLK / NW, LB = (B_BLK + NW - 1) / NW, LPW = LA + LB;
  constexpr int STAGE = (A_BLK + LB * NW) * 64;  // 16-byte chunks per stage
  constexpr bool SWAP = !SCORE;
  static_assert(A_BLK % NW == 0, "the tokens' blocks must divide over the wavefronts");
  static_assert(KB % KG == 0 && (KS == 1 || KS == 2), "one or two k steps per wavefront and slab");
  static_assert(STAGES >= 2 && (STAGES - 1) * LPW + LPW <= 63, "loads in flight must fit the counter");
  static_assert(ACT != ACT_GLU || (TN % 2 == 0), "GLU needs paired column blocks per wave");
  static_assert(!(SCORE && KG > 1), "the score epilogue has no in-workgroup split");

  extern __shared__ u32x4_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = wave / NWT, wloc = wave % NWT;
  const int wm = wloc / WGN, wn = wloc % WGN;
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tiles_m = (p.M + BM - 1) / BM;
  const int logical = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int gsz = p.group_m * tiles_n;
  const int first_m = (logical / gsz) * p.group_m;
  const int gm = min(tiles_m - first_m, p.group_m);
  const int tm = first_m + (logical % gsz) % gm, tn = (logical % gsz) / gm;
  const int m0 = tm * BM, n0 = tn * BN;

  // K range of this split (whole slabs)
  const int kt_total = (p.K + BK - 1) / BK;
  const int kt_per = (kt_total + (int)gridDim.y - 1) / (int)gridDim.y;
  const int kt0 = blockIdx.y * kt_per;
  const int nk = min(kt_total, kt0 + kt_per) - kt0;

  // ---- the LPW blocks this wavefront moves per slab: block b = wave + i NW of the stage
  // Row-major A: one load instruction covers 64 / CH rows x the slab's CH 16-byte chunks of each
  // (32-deep slabs: 16 rows x 64 contiguous bytes = 16 cache lines; 64-deep: 8 rows x 128 bytes
  // = 8 lines) instead of 32 rows x 32 bytes; the chunks are placed so that the fragment reads
  // stay free of bank conflicts.
  constexpr bool rowsN = !A_TILED && !DUAL && (KB == 2 || KB == 4);
  constexpr int CH = 2 * KB, RPI = 64 / CH;   // chunks per row and slab, rows per instruction
  // chunk swizzle of row rowl of block kb: 16 consecutive lanes of a fragment read (rows r..r+15,
  // one chunk number) must fall into 16 different 16-byte bank groups
  auto swz = [](int rowl, int kb) { return KB == 2 ? ((rowl >> 2) & 3) : ((rowl >> 1) | ((kb & 1) << 2)); };
  const char* src[LPW];
  const char* a_row[LA];   // row-major A: start of the lane's row (substitute for chunks past K)
  int a_col[LA];           // row-major A: column of the lane's chunk inside the slab
  const int mrb_last = (p.M + 31) / 32 - 1, nrb_last = (p.N + 31) / 32 - 1;
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    const int b = wave + i * NW;
    const int s = b / ((BM / 32) * KB), rb = (b / KB) % (BM / 32), kb = b % KB;
    const char* base = (DUAL && s) ? (const char*)p.A1 : (const char*)p.A;
    if (A_TILED) {
      int grb = m0 / 32 + rb;
      grb = grb <= mrb_last ? grb : mrb_last;
      src[i] = base + (((int64_t)grb * (p.lda / 16) + (int64_t)kt0 * KB + kb) * 64 + lane) * 16;
      a_row[i] = nullptr; a_col[i] = 0;
    } else {
      int row = m0 + rb * 32 + (lane & 31);
      a_col[i] = kb * 16 + (lane >> 5) * 8;
      if (rowsN) {
        // block (rb, kb) holds rows RPI kb .. RPI kb + RPI - 1 of the row block with all CH
        // chunks of the slab: lane = CH rowl + position, chunk = position ^ swz
        const int rowl = lane / CH;
        row = m0 + rb * 32 + kb * RPI + rowl;
        a_col[i] = ((lane % CH) ^ swz(rowl, kb)) * 8;
      }
      row = row < p.M ? row : p.M - 1;
      a_row[i] = base + (int64_t)row * p.lda * 2;
      src[i] = a_row[i] + ((int64_t)kt0 * BK + a_col[i]) * 2;
    }
  }
  // LDS offset (16-byte units) of the lane's A fragment inside a row block's KB blocks, per k block
  int a_frag[2];   // per k step of the wavefront inside a slab
  a_frag[0] = lane; a_frag[1] = 64 + lane;
  if (rowsN) {
    const int r = lane & 31, c = lane >> 5, kbr = r / RPI, rowl = r % RPI;
#pragma unroll
    for (int ls = 0; ls < KS; ++ls)
      a_frag[ls] = kbr * 64 + rowl * CH + ((2 * (kg * KS + ls) + c) ^ swz(rowl, kbr));
  }
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    const int b = wave + i * NW;
    const int rb = min(b / KB, BN / 32 - 1), kb = b % KB;
    int grb = n0 / 32 + rb;
    grb = grb <= nrb_last ? grb : nrb_last;
    src[LA + i] = (const char*)p.Bt + (((int64_t)grb * (p.ldb / 16) + (int64_t)kt0 * KB + kb) * 64 + lane) * 16;
  }

  // Part q of KS of the loads of slab rel (spread over the k steps, between the MFMAs)
  auto issue_part = [&](int rel, int stage, int q) {
    u32x4_t* st = smem + stage * STAGE;
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      if (i * KS / LPW != q) continue;
      const char* g;
      int slot;
      if (i < LA) {
        slot = wave + i * NW;
        if (A_TILED) {
          g = src[i] + (int64_t)rel * (KB * 1024);
        } else {
          // a chunk past K reads the start of the row instead: the weights are zero there
          g = ((kt0 + rel) * BK + a_col[i] < p.K) ? src[i] + (int64_t)rel * (BK * 2) : a_row[i];
        }
      } else {
        slot = A_BLK + wave + (i - LA) * NW;
        g = src[i] + (int64_t)rel * (KB * 1024);
      }
      __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)(st + slot * 64), 16, 0, 0);
    }
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // Residual stream of an un-activated product: the accumulators start from it (same lane
  // layout as the store epilogue: row lane & 31, columns 8 g + 4 (lane >> 5) + 0..3 of each
  // tile), so its loads overlap the filling of the ring instead of forming one dependent
  // round trip per tile between the last product and the stores.  This workgroup alone
  // reads and later writes these elements, so the destination may be the residual buffer.
  if (EPI && ACT == ACT_NONE && !SCORE && SWAP) {
    if (p.resid != nullptr && !p.partial && !p.c0_tiled && kg == 0) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int cb = n0 + wn * WN + j * 32;
        if (cb >= p.N || cb >= p.split_col) continue;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int row = m0 + wm * WM + i * 32 + (lane & 31);
          if (row >= p.M) continue;
          const float* rrow = p.resid + (int64_t)row * p.ldr + cb + 4 * (lane >> 5);
#pragma unroll
          for (int g = 0; g < 4; ++g)
            if (cb + 8 * g + 4 * (lane >> 5) < p.n_store) {
              const float4 r4 = *(const float4*)(rrow + 8 * g);
              acc[i][j][4 * g] = r4.x; acc[i][j][4 * g + 1] = r4.y; acc[i][j][4 * g + 2] = r4.z; acc[i][j][4 * g + 3] = r4.w;
            }
        }
      }
    }
  }

  // Fragment reads run one k step ahead of the MFMAs (two register sets), also across the
  // slab boundary, so LDS traffic overlaps the matrix pipeline instead of following a barrier.
  Frag fa[2][NA][TM], fb[2][TN];
  auto read_frags = [&](int set, int stage, int ls) {
    const int ks = kg * KS + ls;   // this wavefront's k block of the slab
    const u32x4_t* sA = smem + stage * STAGE;
    const u32x4_t* sB = sA + A_BLK * 64;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int s = 0; s < NA; ++s) {
        if (rowsN)
          fa[set][s][i].u = sA[(wm * TM + i) * KB * 64 + a_frag[ls]];
        else
          fa[set][s][i].u = sA[((s * (BM / 32) + wm * TM + i) * KB + ks) * 64 + lane];
      }
#pragma unroll
    for (int jj = 0; jj < TN; ++jj) fb[set][jj].u = sB[((wn * TN + jj) * KB + ks) * 64 + lane];
  };
  auto mfma_step = [&](int set) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int jj = 0; jj < TN; ++jj) {
        const Frag& af = fa[set][DUAL ? (jj & 1) : 0][i];
        if (SWAP)
          acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][jj].v, af.v, acc[i][jj], 0, 0, 0);
        else
          acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, fb[set][jj].v, acc[i][jj], 0, 0, 0);
      }
  };
  // Instruction order of one k step: the memory instructions (first the LDS reads of the next
  // step, then the direct loads) are dealt out evenly between the MFMAs; bursts of memory
  // instructions stall the issuing wavefront and with it the matrix pipeline.
  auto order_step = [&](auto nl) {
    constexpr int nload = decltype(nl)::value;
    constexpr int NR = NA * TM + TN, NM = TM * TN, TOT = NR + nload;
    constexpr int PER = TOT / NM, REM = TOT % NM;
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
  };
  // slab s has landed once at most the loads of the slabs issued after it are outstanding;
  // `last` is the last slab issued so far
  auto wait_landed = [&](int s, int last, auto full) {
    if (decltype(full)::value) {
      wait_vmcnt<(STAGES - 2) * LPW>();
    } else {
      const int later = min(nk - 1, last) - s;
      if (later <= 0) wait_vmcnt<0>();
      else if (later == 1) wait_vmcnt<LPW>();
      else if (later == 2) wait_vmcnt<2 * LPW>();
      else if (later == 3) wait_vmcnt<3 * LPW>();
      else if (later == 4) wait_vmcnt<4 * LPW>();
      else if (later == 5) wait_vmcnt<5 * LPW>();
      else wait_vmcnt<6 * LPW>();
    }
  };
  static_assert(STAGES <= 8, "wait_landed covers up to six slabs in flight behind the awaited one");

  // The wavefront's local k steps n = 0, 1, ... (slab n / KS, step n % KS).  During step n the
  // fragments of step n + 1 are read.  Right after the reads of a slab's last step are issued
  // comes that slab's barrier: it publishes the next slab (whose first read follows) and
  // retires this one, whose stage the loads issued from then on refill STAGES slabs ahead.
  const int nsteps = nk * KS;
  // prologue: with one step per slab all STAGES stages are filled; with two, the last stage gets
  // its first part only (its second part goes out with step 0, like every later slab's)
#pragma unroll
  for (int s = 0; s < STAGES; ++s)
    if (s < nk) {
#pragma unroll
      for (int q = 0; q < KS; ++q)
        if (KS == 1 || s < STAGES - 1 || q == 0) issue_part(s, s, q);
    }
  if (nk > 0) {
    wait_landed(0, KS == 1 ? STAGES - 1 : STAGES - 2, std::false_type{});
    lds_barrier();
    read_frags(0, 0, 0);
    if (KS == 1) {
      // slab 0 is already retired by that read: its barrier
      wait_landed(1, STAGES - 1, std::false_type{});
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
  }
  // One unrolled group of U steps starting at step n0 (n0 % U == 0 keeps register sets and
  // slab-local step numbers static).  FULL: every load referred to exists.
  constexpr int U = 2;
  int slab = 0, stage = 0;   // slab and stage of step n0
  auto group = [&](int n0, auto full) {
    constexpr bool FULL = decltype(full)::value;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ls = KS == 1 ? 0 : u;                 // step inside its slab
      const bool last_of_slab = (ls == KS - 1);
      const int nstage = stage + 1 == STAGES ? 0 : stage + 1;
      // the step being prefetched: (slab, ls + 1) or (slab + 1, 0)
      const int pslab = last_of_slab ? slab + 1 : slab;
      const int pstage = last_of_slab ? nstage : stage;
      const int pls = last_of_slab ? 0 : ls + 1;
      if (FULL || n0 + u < nsteps) {
        read_frags((u + 1) & 1, pstage, pls);   // (past the end: stale data that is never used)
        // Loads: the latest barrier before this step retired slab r (with two steps per slab,
        // r = slab - 1 at step 0, where stage "r = -1" is the last, still empty one); the parts
        // of slab r + STAGES go out with the steps that follow that barrier.
        {
          const int r = KS == 1 ? slab : (ls == 0 ? slab - 1 : slab);
          const int rstage = KS == 1 ? stage : (ls == 0 ? (stage == 0 ? STAGES - 1 : stage - 1) : stage);
          const int q = KS == 1 ? 0 : (ls == 0 ? 1 : 0);
          if (FULL || r + STAGES < nk) issue_part(r + STAGES, rstage, q);
        }
        mfma_step(u & 1);
        if (FULL) {
          if (KS == 1) order_step(std::integral_constant<int, LPW>{});
          else if (ls == 0) order_step(std::integral_constant<int, LPW - (LPW + 1) / 2>{});   // part 1
          else order_step(std::integral_constant<int, (LPW + 1) / 2>{});                        // part 0
        }
        // barrier of slab pslab once the reads of its last step are issued
        if (pls == KS - 1) {
          wait_landed(pslab + 1, pslab + STAGES - 1, full);
          asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        }
      }
      if (last_of_slab) { slab += 1; stage = nstage; }
    }
  };
  int n = 0;
  // FULL while the group's last retired slab r satisfies r + STAGES < nk and the prefetched slab
  // + STAGES - 1 <= nk - 1 (so the fixed wait count is right)
  for (; (n + U - 1) / KS + 1 + STAGES < nk; n += U) group(n, std::true_type{});
  for (; n < nsteps; n += U) group(n, std::false_type{});

  if (KG > 1) {
    // Sum the k groups' accumulators: groups 1 .. KG-1 park theirs in LDS (a lane's 16 bytes of
    // one 32x32 tile quarter, contiguous per wavefront instruction), group 0 adds them in order.
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    constexpr int PER_WAVE = TM * TN * 4 * 64;   // 16-byte chunks parked per wavefront
#pragma unroll 1
    for (int g = 1; g < KG; ++g) {
      if (kg == g) {
        u32x4_t* dst = smem + wloc * PER_WAVE + lane;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const u32x4_t v = {__float_as_uint(acc[i][j][4 * q]), __float_as_uint(acc[i][j][4 * q + 1]),
                                 __float_as_uint(acc[i][j][4 * q + 2]), __float_as_uint(acc[i][j][4 * q + 3])};
              dst[((i * TN + j) * 4 + q) * 64] = v;
            }
      }
      __syncthreads();
      if (kg == 0) {
        const u32x4_t* srcp = smem + wloc * PER_WAVE + lane;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const u32x4_t v = srcp[((i * TN + j) * 4 + q) * 64];
#pragma unroll
              for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += __uint_as_float(v[e]);
            }
      }
      if (g + 1 < KG) __syncthreads();
    }
    if (kg != 0) return;
  }
  if (SCORE) lds_barrier();   // the epilogue reuses the stage memory
  gemm_epilogue<BM, BN, WGM, WGN, ACT, SCORE, EPI>(p, acc, m0, n0, tm, wm, wn, lane, tid & (NWT * 64 - 1), smem);
}

// Sum of fp32 split-K partials [n_split][M][N] (fixed order) -> bf16, tiled or row-major.
__global__ void splitk_reduce_kernel(const float* part, int n_split, int M, int N, int m_pad, void* C, int64_t ldc,
                                     int tiled, int f32_out) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one 8-column chunk each
  const int cpr = N / 8;
  if (id >= (int64_t)m_pad * cpr) return;
  const int row = (int)(id / cpr), c8 = (int)(id % cpr) * 8;
  float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (row < M)
    for (int s = 0; s < n_split; ++s) {
      const float4 a = *(const float4*)(part + ((int64_t)s * M + row) * N + c8);
      const float4 b = *(const float4*)(part + ((int64_t)s * M + row) * N + c8 + 4);
      v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w; v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
    }
  if (f32_out) {
    if (row < M) {
      float* dst = (float*)C + (int64_t)row * ldc + c8;
      *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
      *(float4*)(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
    return;
  }
  const uint4 val = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                               pack_bf16x2(v[6], v[7]));
  if (tiled) {
    const int64_t blk = (int64_t)(row / 32) * (ldc / 16) + c8 / 16;
    *(uint4*)((char*)C + ((blk * 64) + ((c8 >> 3) & 1) * 32 + (row & 31)) * 16) = val;
  } else if (row < M) {
    *(uint4*)((char*)C + ((int64_t)row * ldc + c8) * 2) = val;
  }
}

int launch_splitk_reduce(const float* part, int n_split, int M, int N, int m_pad, void* C, int64_t ldc, int tiled,
                         hipStream_t st, int f32_out) {
  const int64_t n = (int64_t)m_pad * (N / 8);
  if (n <= 0) return 0;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, n_split, M, N,
                     m_pad, C, ldc, tiled, f32_out);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Sum of fp32 split-K partials [n_split][M][ldp] of a whole product (GEMM column order) followed
// by the store epilogue of the large-batch kernel: activation (GeLU, or SwiGLU on (gate, up)
// pairs of 32-column blocks), routing to two destinations, bf16, tiled or row-major.  Used for
// products with few tiles at a few hundred rows, which are split along the reduction to fill
// the machine.  One thread per (row, 8 output columns).
struct SplitEpiArgs {
  const float* part;
  int n_split, M, ldp, n_out, rows;   // rows: rows to write (padded to 32 for tiled destinations)
  int act, act_cols, split_col;
  void* C0;
  void* C1;
  int64_t ldc0, ldc1;
  int c0_tiled, c1_tiled, n_store;
  const float* bias;   // as in GemmArgs
  int bias_cols;
  const float* resid;
  int64_t ldr;
  int out_f32;
};

__global__ void __launch_bounds__(256) splitk_epilogue_kernel(const SplitEpiArgs p) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int cpr = p.n_out / 8;
  if (id >= (int64_t)p.rows * cpr) return;
  const int row = (int)(id / cpr), oc = (int)(id % cpr) * 8;
  const bool glu = p.act == ACT_GLU;
  const bool pair = glu && oc < p.act_cols / 2;
  int c = oc;                                   // GEMM column of the (gate) values
  if (glu) c = pair ? (oc / 32) * 64 + (oc & 31) : oc + p.act_cols / 2;
  float v[8] = {0, 0, 0, 0, 0, 0, 0, 0}, u[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (row < p.M) {
    for (int s = 0; s < p.n_split; ++s) {
      const float* src = p.part + ((int64_t)s * p.M + row) * p.ldp + c;
      const float4 a = *(const float4*)src, b = *(const float4*)(src + 4);
      v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w; v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
      if (pair) {
        const float4 e = *(const float4*)(src + 32), f = *(const float4*)(src + 36);
        u[0] += e.x; u[1] += e.y; u[2] += e.z; u[3] += e.w; u[4] += f.x; u[5] += f.y; u[6] += f.z; u[7] += f.w;
      }
    }
    if (!glu && p.bias != nullptr && c + 7 < p.bias_cols) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += p.bias[c + e];
    }
    if (pair) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = silu_fast(v[e]) * u[e];
    } else if (p.act == ACT_GELU && c < p.act_cols) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = gelu_fast(v[e]);
    }
  }
  char* base;
  int64_t ld;
  int col, tiled;
  const bool to_c0 = oc < p.split_col;
  if (to_c0) { base = (char*)p.C0; ld = p.ldc0; col = oc; tiled = p.c0_tiled; }
  else { base = (char*)p.C1; ld = p.ldc1; col = oc - p.split_col; tiled = p.c1_tiled; }
  if (to_c0 && !tiled && row < p.M && col < p.n_store) {
    if (p.resid != nullptr) {
      const float* r = p.resid + (int64_t)row * p.ldr + col;
      const float4 a = *(const float4*)r, b = *(const float4*)(r + 4);
      v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w; v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
    }
    if (p.out_f32) {
      float* dst = (float*)base + (int64_t)row * ld + col;
      *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
      *(float4*)(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
      return;
    }
  }
  const uint4 val = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                               pack_bf16x2(v[6], v[7]));
  if (tiled) {
    const int64_t blk = (int64_t)(row / 32) * (ld / 16) + col / 16;
    *(uint4*)(base + ((blk * 64) + ((col >> 3) & 1) * 32 + (row & 31)) * 16) = val;
  } else if (row < p.M && col < p.n_store) {
    *(uint4*)(base + ((int64_t)row * ld + col) * 2) = val;
  }
}

int launch_splitk_epilogue(const float* part, int n_split, int ldp, const GemmArgs& g, int act, hipStream_t st) {
  SplitEpiArgs a = {};
  a.part = part; a.n_split = n_split; a.M = g.M; a.ldp = ldp;
  a.n_out = act == ACT_GLU ? g.N - g.act_cols / 2 : g.N;
  a.rows = (g.c0_tiled || g.c1_tiled) ? (g.M + 31) / 32 * 32 : g.M;
  a.act = act; a.act_cols = g.act_cols; a.split_col = g.split_col;
  a.C0 = g.C0; a.C1 = g.C1; a.ldc0 = g.ldc0; a.ldc1 = g.ldc1;
  a.c0_tiled = g.c0_tiled; a.c1_tiled = g.c1_tiled; a.n_store = g.n_store;
  a.bias = g.bias; a.bias_cols = g.bias_cols; a.resid = g.resid; a.ldr = g.ldr; a.out_f32 = g.out_f32;
  if ((a.n_out & 7) || (g.split_col & 7) || (g.act_cols & 63)) return -1;
  const int64_t n = (int64_t)a.rows * (a.n_out / 8);
  if (n <= 0) return 0;
  hipLaunchKernelGGL(splitk_epilogue_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// ------------------------------------------------------------------ host launcher

template <int BM, int BN, int BK, int WGM, int WGN, int KG, int STAGES, int ACT, bool DUAL, bool SCORE, bool A_TILED,
          bool EPI>
static int launch_dl_epi(const GemmArgs& a, int n_split, hipStream_t st) {
  constexpr int NA = DUAL ? 2 : 1;
  constexpr int NWH = WGM * WGN * KG, BBLK = (BN / 32) * (BK / 16);
  constexpr size_t ring = (size_t)STAGES * ((size_t)NA * BM * BK * 2 + (size_t)((BBLK + NWH - 1) / NWH) * NWH * 1024);
  constexpr size_t park = KG > 1 ? (size_t)BM * BN * 4 : 0;   // one k group's accumulators
  constexpr size_t lds = ring > park ? ring : park;
  static_assert(lds <= 160 * 1024, "LDS budget of a CU");
  auto kern = gemm_bf16_dl_kernel<BM, BN, BK, WGM, WGN, KG, STAGES, ACT, DUAL, SCORE, A_TILED, EPI>;
  // The kernel needs more dynamic LDS than the default limit: the attribute is set once per
  // device and instantiation.  The only state kept is this set-once bit mask (one bit per
  // device ordinal); setting the attribute twice from racing first calls is harmless.
  static std::atomic<uint64_t> configured{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return -1;
  const uint64_t bit = 1ull << (dev & 63);
  if (dev >= 64 || !(configured.load(std::memory_order_acquire) & bit)) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return -1;
    if (dev < 64) configured.fetch_or(bit, std::memory_order_release);
  }
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(tiles, n_split), dim3(WGM * WGN * KG * 64), lds, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <int BM, int BN, int BK, int WGM, int WGN, int KG, int STAGES, int ACT, bool DUAL, bool SCORE, bool A_TILED>
static int launch_dl_cfg(const GemmArgs& a, int n_split, hipStream_t st) {
  // (the calibration product, the gated products and the two-operand product take no additions)
  if constexpr (!SCORE && !DUAL && ACT != ACT_GLU) {
    if (a.bias != nullptr || a.resid != nullptr || a.out_f32)
      return launch_dl_epi<BM, BN, BK, WGM, WGN, KG, STAGES, ACT, DUAL, SCORE, A_TILED, true>(a, n_split, st);
  } else {
    if (a.bias != nullptr || a.resid != nullptr || a.out_f32) return -1;
  }
  return launch_dl_epi<BM, BN, BK, WGM, WGN, KG, STAGES, ACT, DUAL, SCORE, A_TILED, false>(a, n_split, st);
}

template <int BM, int BN, int BK, int WGM, int WGN, int KG, int STAGES>
static int launch_dl_shape(const GemmArgs& a, int act, int n_split, hipStream_t st) {
  const bool dual = a.A1 != nullptr;
  const bool at = a.a_tiled != 0;
  if (act == ACT_NONE)
    return at ? launch_dl_cfg<BM, BN, BK, WGM, WGN, KG, STAGES, ACT_NONE, false, false, true>(a, n_split, st)
              : launch_dl_cfg<BM, BN, BK, WGM, WGN, KG, STAGES, ACT_NONE, false, false, false>(a, n_split, st);
  if (act == ACT_GELU)
    return at ? launch_dl_cfg<BM, BN, BK, WGM, WGN, KG, STAGES, ACT_GELU, false, false, true>(a, 1, st)
              : launch_dl_cfg<BM, BN, BK, WGM, WGN, KG, STAGES, ACT_GELU, false, false, false>(a, 1, st);
  if constexpr (BN / WGN >= 64 && (BN / WGN / 32) % 2 == 0) {
    if (act == ACT_GLU && !dual)
      return at ? launch_dl_cfg<BM, BN, BK, WGM, WGN, KG, STAGES, ACT_GLU, false, false, true>(a, 1, st)
                : launch_dl_cfg<BM, BN, BK, WGM, WGN, KG, STAGES, ACT_GLU, false, false, false>(a, 1, st);
    if constexpr ((2 * (BM / 32) * (BK / 16)) % (WGM * WGN * KG) == 0) {
      // two left operands double the A part of a stage: fewer stages where that keeps two
      // workgroups per CU (80 KiB each)
      // (a 256 x 256 tile runs one workgroup per CU anyway: it keeps its three stages, 144 KiB)
      constexpr int DST = (BM * BN >= 256 * 256) ? STAGES
                          : (((size_t)STAGES * (2 * BM + BN) * BK * 2 > 80 * 1024 && STAGES > 2) ? 2 : STAGES);
      if constexpr ((size_t)DST * (2 * BM + BN) * BK * 2 <= 160 * 1024) {
        if (act == ACT_GLU && dual && at)
          return launch_dl_cfg<BM, BN, BK, WGM, WGN, KG, DST, ACT_GLU, true, false, true>(a, 1, st);
      }
    }
  }
  return -1;
}

int bf16_score_tile_m() { return 256; }

int launch_gemm_bf16(const GemmArgs& a, int act, bool score, int shape, int n_split, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0) return 0;
  if (score) {
    // calibration: row-major tokens, column sums of the activations in the epilogue
    if (a.a_tiled) return -1;
    if (act == ACT_GELU) return launch_dl_cfg<256, 256, 32, 2, 4, 1, 3, ACT_GELU, false, true, false>(a, 1, st);
    if (act == ACT_GLU) return launch_dl_cfg<256, 256, 32, 2, 4, 1, 3, ACT_GLU, false, true, false>(a, 1, st);
    return -1;
  }
  switch (shape) {
    case GEMM_256x128: return launch_dl_shape<256, 128, 32, 2, 2, 1, 3>(a, act, n_split, st);
    case GEMM_128x128: return launch_dl_shape<128, 128, 32, 2, 2, 1, 3>(a, act, n_split, st);
    case GEMM_128x128_KSPLIT: return launch_dl_shape<128, 128, 64, 2, 2, 2, 4>(a, act, n_split, st);
    case GEMM_256x256: return launch_dl_shape<256, 256, 32, 2, 4, 1, 3>(a, act, n_split, st);
    case GEMM_256x320: return launch_dl_shape<256, 320, 32, 4, 2, 1, 3>(a, act, n_split, st);
    case GEMM_128x320: return launch_dl_shape<128, 320, 32, 2, 2, 1, 3>(a, act, n_split, st);
    case GEMM_256x256_W64: return launch_dl_shape<256, 256, 32, 4, 2, 1, 3>(a, act, n_split, st);
  }
  return -1;
}

}  // namespace ffsplit
