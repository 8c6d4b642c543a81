// Internal: the private layout of the packed split and of the per-call scratch.
// Pure host arithmetic on the descriptor, so that no call ever has to read
// device memory to find its way around a split.
#pragma once
#include "../../include/ffsplit.h"
#include <stddef.h>
#include <stdint.h>

namespace ffsplit {

inline int round_up(int v, int q) { return (v + q - 1) / q * q; }
inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// All matrices of the split are stored "neuron-major" (transposed, K-contiguous),
// zero-padded: a padded neuron has a zero up column and a zero down row, and
// gelu(0) = silu(0)*0 = 0, so padding changes no result.  fp32: row-major with
// the given row length.  bf16: the 32x16-block tiled layout of gemm_bf16.hip,
// rows padded to 32 and the row length (K) to 64.
//   B1t [n1, d]      rows: heavy W1^T (SwiGLU: 32-row blocks gate/up interleaved),
//                    then LOWRANK: Pg^T, P1^T ;  DENSE: the remainder's W1^T likewise
//   Q1t [n_up*mp, rp] LOWRANK: Q1^T (SwiGLU: Qg^T / Q1^T interleaved in 32-row blocks)
//   P2t [rp, mp]      LOWRANK: P2^T
//   B4t [d, k4]       columns: heavy W2^T (kp), then Q2^T (rp) or the remainder's W2^T (mp)
struct Layout {
  int n_up;   // 1 GeLU, 2 SwiGLU
  int esz;
  int kp, rp, mp;
  int k4;     // K of the last product
  int n1;     // rows of B1t
  int tiled;  // bf16: tiled layout
  int dk;     // row length of B1t (d_model, padded to 64 when tiled)
  int dn;     // rows of B4t (d_model, padded to 32 when tiled)
  size_t off_b1, off_q1, off_p2, off_b4;
  // INT4 remainder (decode layout, see int4.hip)
  int jp16, jp128, kp128, groups;
  size_t off_i4[3], off_s4[3];       // nibbles / scales of gate(W1), Wg, W2
  size_t off_hv[3];                  // heavy bf16 blocks in decode order
  // W3H8 (quant.hip): four quantised matrices, 0 heavy up/gate rows (int8), 1 remainder up/gate
  // rows (int3), 2 heavy down columns (int8), 3 remainder down columns (int3)
  size_t off_qc[4], off_qs[4];       // codes / fp16 scales
  size_t total_bytes;
};

// quantised tiled blocks: 32 rows x 64 reduction elements
inline size_t qblock_bytes(int bits) { return bits == 8 ? 2048 : 768; }

inline Layout make_layout(const ffsplit_desc_t& d) {
  Layout L = {};
  L.n_up = d.act == FFSPLIT_ACT_SWIGLU ? 2 : 1;
  L.esz = d.dtype == FFSPLIT_BF16 ? 2 : 4;
  const int m = d.d_ff - d.k;
  L.kp = round_up(d.k, 64);
  const bool lr = d.rem_kind == FFSPLIT_REM_LOWRANK && m > 0;
  const bool dn = d.rem_kind == FFSPLIT_REM_DENSE && m > 0;
  const bool i4 = d.rem_kind == FFSPLIT_REM_INT4;
  const bool q38 = d.rem_kind == FFSPLIT_REM_W3H8;
  L.rp = lr ? round_up(d.rank, 64) : 0;
  L.mp = (lr || dn || q38) ? round_up(m, 64) : 0;
  L.k4 = L.kp + (lr ? L.rp : 0) + ((dn || q38) ? L.mp : 0);
  L.n1 = L.n_up * L.k4;
  size_t off = 0;
  L.tiled = d.dtype == FFSPLIT_BF16;
  L.dk = L.tiled ? round_up(d.d_model, 64) : d.d_model;
  L.dn = L.tiled ? round_up(d.d_model, 32) : d.d_model;
  if (q38) {
    // same padded counts and row order as the DENSE layout, so that expanding gives its image
    L.groups = d.d_model / 128;
    const int rows[4] = {L.n_up * L.kp, L.n_up * L.mp, L.dn, L.dn};
    const int ks[4] = {L.dk, L.dk, L.kp, L.mp};
    for (int i = 0; i < 4; ++i) {
      const int bits = (i & 1) ? 3 : 8;
      L.off_qc[i] = off; off = align256(off + (size_t)(rows[i] / 32) * (ks[i] / 64) * qblock_bytes(bits));
      // up / gate: one scale per (row, group of 128 inputs); down: per (group of 128 outputs, neuron)
      L.off_qs[i] = off;
      off = align256(off + (i < 2 ? (size_t)rows[i] * L.groups * 2 : (size_t)(L.dn / 128) * ks[i] * 2));
    }
  } else if (!i4) {
    L.off_b1 = off; off = align256(off + (size_t)L.n1 * L.dk * L.esz);
    L.off_q1 = off; if (lr) off = align256(off + (size_t)L.n_up * L.mp * L.rp * L.esz);
    L.off_p2 = off; if (lr) off = align256(off + (size_t)L.rp * L.mp * L.esz);
    L.off_b4 = off; off = align256(off + (size_t)L.dn * L.k4 * L.esz);
  } else {
    L.groups = d.d_model / 128;
    L.jp16 = round_up(m, 16);
    L.jp128 = round_up(m, 128);
    L.kp = round_up(d.k, 16);
    L.kp128 = round_up(d.k, 128);
    L.k4 = L.kp; L.n1 = 0;
    for (int w = 0; w < 3; ++w) {
      const bool used = (w != 1) || L.n_up == 2;
      const size_t nib = w == 2 ? (size_t)L.jp128 * d.d_model / 2 : (size_t)L.jp16 * d.d_model / 2;
      const size_t sc = w == 2 ? (size_t)L.jp128 * L.groups * 2 : (size_t)L.jp16 * L.groups * 2;
      const size_t hv = w == 2 ? (size_t)L.kp128 * d.d_model * 2 : (size_t)L.kp * d.d_model * 2;
      L.off_i4[w] = off; if (used) off = align256(off + nib);
      L.off_s4[w] = off; if (used) off = align256(off + sc);
      L.off_hv[w] = off; if (used) off = align256(off + hv);
    }
  }
  L.total_bytes = off > 0 ? off : 256;
  return L;
}

struct ScoreWs {
  int n_gemm, n_out, tiles_m, dk;
  size_t off_wt, wt_bytes, off_p2, off_p1, total_bytes;
};

inline ScoreWs make_score_ws(const ffsplit_desc_t& d, int64_t T) {
  ScoreWs w = {};
  const int n_up = d.act == FFSPLIT_ACT_SWIGLU ? 2 : 1;
  const int esz = d.dtype == FFSPLIT_BF16 ? 2 : 4;
  const int tile_m = d.dtype == FFSPLIT_BF16 ? 256 : 64;
  w.n_out = round_up(d.d_ff, 64);
  w.n_gemm = n_up * w.n_out;
  w.tiles_m = (int)((T + tile_m - 1) / tile_m);
  w.off_wt = 0;
  w.dk = d.dtype == FFSPLIT_BF16 ? round_up(d.d_model, 64) : d.d_model;
  w.wt_bytes = align256((size_t)w.n_gemm * w.dk * esz);
  w.off_p2 = w.wt_bytes;
  const size_t pb = align256((size_t)(w.tiles_m > 0 ? w.tiles_m : 1) * w.n_out * 4);
  w.off_p1 = w.off_p2 + pb;
  w.total_bytes = w.off_p1 + pb;
  return w;
}

// A few hundred rows (above the weight-streaming kernels, up to 1024): a product with fewer than
// 128 tiles of 128 x 128 is split along its reduction into about 256 workgroups (at least 256
// reduction elements each); its fp32 partials then take the epilogue in a second launch.
inline int mid_split(int64_t T, int N, int K) {
  const int tiles = (int)((T + 127) / 128) * ((N + 127) / 128);
  if (tiles <= 0 || tiles >= 128) return 1;
  int sp = 256 / tiles;
  if (sp > K / 256) sp = K / 256;
  if (sp > 16) sp = 16;
  return sp > 1 ? sp : 1;
}

// fp32 path: a product with few 64 x 64 tiles (its workgroups each walk the whole reduction in
// 16-deep slabs, one after the other) is split along the reduction into up to about 192
// workgroups of at least 64 reduction elements; fp32 partials, then one summing launch that
// also applies bias / activation / routing.
inline int f32_split(int64_t T, int N, int K) {
  const int tiles = (int)((T + 63) / 64) * ((N + 63) / 64);
  if (tiles <= 0 || tiles >= 96 || K < 128) return 1;
  int sp = 192 / tiles;
  if (sp > K / 64) sp = K / 64;
  if (sp > 32) sp = 32;
  return sp > 1 ? sp : 1;
}

struct FwdWs {
  size_t off_cat, off_t, off_h2, off_kpart;
  size_t kpart_bytes;   // bytes of split-K scratch at off_kpart (65..1024 rows: checked before use)
  int t_pad;       // rows of the intermediates (T, padded to 32 when tiled)
  int g3_split;    // split-K factor of the h2 * P2 product
  int g3_wide;     // that product has enough tiles for 256x128 tiles (else: in-workgroup K split)
  // INT4 decode scratch
  size_t off_h, off_part, off_cnt;
  int n_split;
  // INT4 with many tokens: bf16 image of the split in the DENSE layout, then that chain's scratch
  int i4_prefill;
  size_t off_img, off_dense;
  size_t total_bytes;
};

// INT4 remainder: up to this many tokens take the weight-streaming decode kernels, 16 tokens
// per pass; beyond it the weights are expanded to bf16 once and the dense chain runs
// (expanding plus the chain at that size costs about as much as 12 passes).
constexpr int INT4_DECODE_MAX_T = 192;
// W3H8: up to this many tokens stream the packed codes, 32 tokens per pass; beyond it they are
// expanded (four passes cost less than expanding plus the chain at that size)
constexpr int W3H8_DECODE_MAX_T = 128;

// The fused middle products (ffn2_fused.hip) serve un-gated bf16 layers of padded rank 512 from
// 8192 tokens on.  With fewer tokens its 128-row tiles have to split the neurons over more than
// four workgroups to fill the machine, and the fp32 partial sums of those ranges cost more than
// not storing h2 saves (measured at the OPT-1.3B shape: 4096 tokens 132 against 128 us per
// forward, 7168 equal, 8192 220 against 250, 16384 421 against 445).
inline bool ffn2_fused_applies(const Layout& L, int64_t T) {
  return L.tiled && L.n_up == 1 && L.rp == 512 && L.mp >= 64 && T >= 8192;
}

inline size_t build_ws_bytes(const ffsplit_desc_t& d) { return align256((size_t)8 * d.d_ff) + 256; }

FwdWs make_fwd_ws(const ffsplit_desc_t& d, const Layout& L, int64_t T);

}  // namespace ffsplit
