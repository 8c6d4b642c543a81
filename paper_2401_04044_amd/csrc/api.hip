// C ABI of libffsplit (declared in include/ffsplit.h): host-side validation,
// the private packed-split layout, and the launch sequences of the four calls.
#include "../../include/ffsplit.h"
#include "layout.h"
#include "prep.h"
#include "int4.h"
#include "quant.h"
#include "factor.h"

using namespace ffsplit;

namespace {

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

int check_desc(const ffsplit_desc_t* d, bool need_split_fields) {
  if (!d) return FFSPLIT_E_NULLPTR;
  if (d->d_model <= 0 || d->d_ff <= 0) return FFSPLIT_E_BADDESC;
  if (d->act != FFSPLIT_ACT_GELU && d->act != FFSPLIT_ACT_SWIGLU) return FFSPLIT_E_BADDESC;
  if (d->dtype != FFSPLIT_F32 && d->dtype != FFSPLIT_BF16) return FFSPLIT_E_BADDESC;
  if (d->d_model % 8 != 0) return FFSPLIT_E_BADSHAPE;
  if (!need_split_fields) return FFSPLIT_OK;
  if (d->rem_kind < FFSPLIT_REM_NONE || d->rem_kind > FFSPLIT_REM_W3H8) return FFSPLIT_E_BADDESC;
  if (d->k < 0 || d->k > d->d_ff) return FFSPLIT_E_BADSHAPE;
  const int m = d->d_ff - d->k;
  if (d->rem_kind == FFSPLIT_REM_LOWRANK && m > 0) {
    if (d->rank <= 0) return FFSPLIT_E_BADSHAPE;
    if (d->rank > (d->d_model < m ? d->d_model : m)) return FFSPLIT_E_BADSHAPE;
  }
  if (d->rem_kind == FFSPLIT_REM_INT4 || d->rem_kind == FFSPLIT_REM_W3H8) {
    if (d->group <= 0 || d->group % 32 != 0 || d->d_model % d->group != 0) return FFSPLIT_E_BADSHAPE;
    if (d->dtype != FFSPLIT_BF16) return FFSPLIT_E_UNSUPPORTED;
    if (d->group != 128 || d->d_model % 128 != 0) return FFSPLIT_E_UNSUPPORTED;
  }
  return FFSPLIT_OK;
}

inline int act_of(const ffsplit_desc_t* d) { return d->act == FFSPLIT_ACT_SWIGLU ? ACT_GLU : ACT_GELU; }

#define FFS_TRY(expr)                      \
  do {                                     \
    if ((expr) != 0) return FFSPLIT_E_HIP; \
  } while (0)

}  // namespace

// The chained products of one forward call for the NONE / DENSE / LOWRANK layouts (sp: packed
// split, ws: scratch laid out by w).  Also the large-batch path of the int4 remainder, which
// first expands its weights to a DENSE image.
static int forward_chain(const ffsplit_desc_t* d, const Layout& L, const FwdWs& w, const char* sp, const void* X, int M,
                         void* Y, void* Y_heavy, void* Y_rem, const Epilogue& ep, char* ws, hipStream_t st) {
  const int bf16 = d->dtype == FFSPLIT_BF16;
  const int esz = bf16 ? 2 : 4;
  const int act = act_of(d);
  const bool glu = act == ACT_GLU;
  const int dm = d->d_model, k = d->k, m = d->d_ff - d->k;
  char* cat = ws + w.off_cat;    // [T, k4]  = [h1 | t2] (or [h1 | h_rest] for DENSE)
  char* tbuf = ws + w.off_t;     // [T, n_up*rp]
  char* h2 = ws + w.off_h2;      // [T, mp]
  const bool rem_lr = d->rem_kind == FFSPLIT_REM_LOWRANK && m > 0;
  const bool rem_dense = d->rem_kind == FFSPLIT_REM_DENSE && m > 0;
  // Column offset inside a K-contiguous buffer: elements (row-major) or whole 16-wide
  // k blocks of 1 KiB (tiled).
  auto koff_bytes = [&](int koff) -> size_t { return L.tiled ? (size_t)(koff / 16) * 1024 : (size_t)koff * esz; };
  // small batches are bound by streaming the weights: dedicated kernels
  const bool small_m = bf16 && M <= SKINNY_MAX_M;
  auto run = [&](GemmArgs& g, int a, int shape, int n_split) -> int {
    if (g.group_m <= 0) g.group_m = 8;
    g.m_pad = w.t_pad;
    if (!bf16) {
      // few tiles: split the reduction, bias / activation / routing with the sum (never beyond
      // the scratch the workspace was sized with: the plain launch is always valid)
      const int sp = (g.partial || g.A1) ? 1 : f32_split(M, g.N, g.K);
      if (sp > 1 && (size_t)sp * M * g.N * 4 <= w.kpart_bytes) {
        float* part = (float*)(ws + w.off_kpart);
        GemmArgs gp = g;
        gp.partial = 1; gp.C0 = part; gp.ldc0 = g.N; gp.split_col = g.N; gp.act_cols = 0;
        gp.bias = nullptr; gp.bias_cols = 0; gp.resid = nullptr; gp.out_f32 = 0;
        if (launch_gemm_f32(gp, ACT_NONE, false, st, sp) != 0) return -1;
        return launch_splitk_epilogue_f32(part, sp, g.N, g, a, st);
      }
      return launch_gemm_f32(g, a, false, st, n_split);
    }
    if (small_m && !g.partial && (g.N & 31) == 0) return launch_skinny_bf16(g, a, (float*)(ws + w.off_kpart), st);
    if (!small_m && M <= 1024 && !g.partial && !g.A1) {
      // a few hundred rows and few tiles: split the reduction, epilogue in a second launch
      const int sp = mid_split(M, g.N, g.K);
      const int ldp = round_up(g.N, 32);
      // (never beyond the scratch the workspace was sized with: the plain launch is always valid)
      if (sp > 1 && (size_t)sp * M * ldp * 4 <= w.kpart_bytes) {
        float* part = (float*)(ws + w.off_kpart);
        GemmArgs gp = g;
        gp.partial = 1; gp.C0 = part; gp.ldc0 = ldp; gp.split_col = ldp; gp.act_cols = 0;
        gp.c0_tiled = 0; gp.c1_tiled = 0;
        gp.bias = nullptr; gp.bias_cols = 0; gp.resid = nullptr; gp.out_f32 = 0;   // applied with the sum
        if (launch_gemm_bf16(gp, ACT_NONE, false, GEMM_128x128, sp, st) != 0) return -1;
        return launch_splitk_epilogue(part, sp, ldp, g, a, st);
      }
    }
    return launch_gemm_bf16(g, a, false, shape, n_split, st);
  };
  const int big_m = M > 1024;   // 256-row tiles only pay off with enough rows
  // Share (percent) of the CU slots that 256x256 tiles keep busy: one workgroup per CU, whole
  // rounds of 256.  Measured: where that share is high the large tile beats the smaller ones
  // by 10-25 % (its main loop reads LDS half as often per MFMA), below about half it loses.
  auto fill256 = [](int m, int n) -> int {
    const int tiles = ((m + 255) / 256) * ((n + 255) / 256);
    return tiles > 0 ? 100 * tiles / (256 * ((tiles + 255) / 256)) : 0;
  };

  // G1: X * [W1h | P1] (SwiGLU: [gate/up heavy pairs | Pg | P1]) -> h1 (activated) and t
  if (L.n1 > 0) {
    GemmArgs g = {};
    g.A = X; g.lda = dm; g.Bt = sp + L.off_b1; g.ldb = L.dk;
    g.M = M; g.N = L.n1; g.K = dm;
    const int acted = rem_dense ? (L.kp + L.mp) : L.kp;   // neurons activated in this product
    g.act_cols = L.n_up * acted;
    g.split_col = acted;
    g.C0 = cat; g.ldc0 = L.k4; g.c0_tiled = L.tiled;
    g.C1 = tbuf; g.ldc1 = (int64_t)L.n_up * L.rp; g.c1_tiled = L.tiled;
    g.group_m = 1;   // X is the large operand: its row tiles stay within one XCD
    g.bias = ep.b1; g.bias_cols = ep.b1 ? acted : 0;   // the activated neurons' biases (packed order)
    // (few tiles: eight wavefronts on 64-deep slabs, whose row-major gather takes whole cache lines)
    int wide = fill256(M, L.n1) >= 50 ? GEMM_256x256 : (L.n1 >= 4096 ? GEMM_256x128 : GEMM_128x128_KSPLIT);
    // A product with fewer 256 x 256 tiles than CUs takes one tile's time whatever the count: where
    // 128 x 320 tiles still fit one round, each CU's share is 0.63 of that (C5: 144 -> 224 tiles,
    // 128 -> 116 us).  Not for gated layers (a wave tile of five column blocks cannot hold pairs).
    if (!glu && wide == GEMM_256x256) {
      const int t256 = ((M + 255) / 256) * ((L.n1 + 255) / 256), t320 = ((M + 127) / 128) * ((L.n1 + 319) / 320);
      if (t256 <= 256 && t320 <= 256) wide = GEMM_128x320;
    }
    FFS_TRY(run(g, act, big_m ? wide : GEMM_128x128, 1));
  }
  // G2 + G3 in one launch where the rank allows it (no neuron bias: that epilogue is G2's)
  bool fused_mid = false;
  if (rem_lr && bf16 && ffn2_fused_applies(L, M) && ep.b1 == nullptr) {
    const int sp2 = ffn2_fused_splits(M, L.mp);
    if ((size_t)sp2 * M * L.rp * 4 <= w.kpart_bytes) {
      float* part = (float*)(ws + w.off_kpart);
      const int rc = launch_ffn2_fused(tbuf, (int64_t)L.n_up * L.rp, sp + L.off_q1, L.rp, sp + L.off_p2, L.mp, M, L.mp,
                                       L.rp, part, sp2, st);
      if (rc < 0) return FFSPLIT_E_HIP;
      if (rc == 0) {
        FFS_TRY(launch_splitk_reduce(part, sp2, M, L.rp, w.t_pad, cat + koff_bytes(L.kp), L.k4, L.tiled, st, 0));
        fused_mid = true;
      }
    }
  }
  if (rem_lr && !fused_mid) {
    // G2: t * Q1 -> activation -> h2
    GemmArgs g = {};
    g.A = tbuf; g.lda = (int64_t)L.n_up * L.rp; g.a_tiled = L.tiled;
    if (glu) g.A1 = tbuf + koff_bytes(L.rp);
    g.Bt = sp + L.off_q1; g.ldb = L.rp;
    g.M = M; g.N = L.n_up * L.mp; g.K = L.rp;
    g.act_cols = g.N; g.split_col = L.mp;
    g.C0 = h2; g.ldc0 = L.mp; g.c0_tiled = L.tiled;
    g.bias = ep.b1 ? ep.b1 + L.kp : nullptr; g.bias_cols = ep.b1 ? L.mp : 0;   // the remainder neurons' biases
    // (a short reduction leaves a 256x256 tile's epilogue uncovered: one workgroup per CU)
    int g2s = (!glu && g.K >= 1024 && fill256(M, g.N) >= 90) ? GEMM_256x256 : GEMM_256x128;
    // two left operands: 256 x 256 tiles with wave tiles of 64 x 128 read each token fragment for
    // four weight blocks instead of two (the Llama shape: 231 -> 200 us)
    if (glu && g.K >= 1024 && fill256(M, g.N) >= 80) g2s = GEMM_256x256_W64;
    FFS_TRY(run(g, act, big_m ? g2s : GEMM_128x128, 1));
    // G3: h2 * P2 -> t2 into cat[:, kp:]  (long reduction: split-K, fixed-order sum)
    g = {};
    g.A = h2; g.lda = L.mp; g.a_tiled = L.tiled;
    g.Bt = sp + L.off_p2; g.ldb = L.mp;
    g.M = M; g.N = L.rp; g.K = L.mp;
    g.split_col = L.rp;
    g.group_m = 1;   // h2 is the large operand
    if (w.g3_split > 1 && !small_m) {
      float* part = (float*)(ws + w.off_kpart);
      g.partial = 1; g.C0 = part; g.ldc0 = L.rp;
      int g3s = big_m ? (w.g3_wide ? GEMM_256x128 : GEMM_128x128_KSPLIT) : GEMM_128x128;
      if (w.g3_wide == 2) g3s = GEMM_256x320;
      if (w.g3_wide == 3) g3s = GEMM_256x256;
      FFS_TRY(run(g, ACT_NONE, g3s, w.g3_split));
      FFS_TRY(launch_splitk_reduce(part, w.g3_split, M, L.rp, w.t_pad, cat + koff_bytes(L.kp), L.k4, L.tiled, st,
                                   bf16 ? 0 : 1));
    } else {
      g.C0 = cat + koff_bytes(L.kp); g.ldc0 = L.k4; g.c0_tiled = L.tiled;
      FFS_TRY(run(g, ACT_NONE, big_m ? GEMM_256x128 : GEMM_128x128, 1));
    }
  }
  // G4: [h1 | t2] * [W2h ; Q2] -> Y   (one fp32 accumulation, one rounding: Eq. 2's sum)
  auto down = [&](void* out, int koff, int klen, bool with_ep) -> int {
    GemmArgs g = {};
    g.A = cat + koff_bytes(koff); g.lda = L.k4; g.a_tiled = L.tiled;
    g.Bt = sp + L.off_b4 + koff_bytes(koff); g.ldb = L.k4;
    g.M = M; g.N = dm; g.K = klen;
    g.split_col = dm; g.C0 = out; g.ldc0 = dm; g.n_store = dm;
    if (with_ep) {   // output bias, residual stream, fp32 destination: Y only
      g.bias = ep.b2; g.bias_cols = ep.b2 ? dm : 0;
      g.resid = ep.resid; g.ldr = dm; g.out_f32 = bf16 ? ep.out_f32 : 0;
    }
    int shp = (big_m && fill256(M, dm) >= 90) ? GEMM_256x256 : GEMM_128x128;
    // 256 x 320 tiles where they fill whole rounds of the 256 CUs and 256 x 256 tiles do not
    // (C5: d_model 5120 = 16 x 320, 4096 rows: exactly 256 tiles; 107 -> 83 us)
    if (big_m && shp == GEMM_128x128 && dm % 320 == 0) {
      const int t320 = ((M + 255) / 256) * (dm / 320);
      if (100 * t320 / (256 * ((t320 + 255) / 256)) >= 90) shp = GEMM_256x320;
    }
    return run(g, ACT_NONE, shp, 1);
  };
  if (L.k4 > 0) {
    FFS_TRY(down(Y, 0, L.k4, true));
  } else if (ep.b2 || ep.resid || (bf16 && ep.out_f32)) {
    return FFSPLIT_E_UNSUPPORTED;   // an empty layer with an epilogue: nothing to fuse it into
  } else {
    FFS_TRY(launch_fill_zero(Y, (size_t)M * dm * esz, st));
  }
  if (Y_heavy) {
    if (L.kp > 0) FFS_TRY(down(Y_heavy, 0, L.kp, false));
    else FFS_TRY(launch_fill_zero(Y_heavy, (size_t)M * dm * esz, st));
  }
  if (Y_rem) {
    if (L.k4 > L.kp) FFS_TRY(down(Y_rem, L.kp, L.k4 - L.kp, false));
    else FFS_TRY(launch_fill_zero(Y_rem, (size_t)M * dm * esz, st));
  }
  (void)k;
  return FFSPLIT_OK;
}

extern "C" {

const char* ffsplit_status_string(int s) {
  switch (s) {
    case FFSPLIT_OK: return "ok";
    case FFSPLIT_E_NULLPTR: return "required pointer is NULL";
    case FFSPLIT_E_BADDESC: return "invalid descriptor field";
    case FFSPLIT_E_BADSHAPE: return "inconsistent shape (k, rank, group, d_model or T)";
    case FFSPLIT_E_ALIGN: return "pointer not 16-byte aligned";
    case FFSPLIT_E_WORKSPACE: return "workspace missing or too small";
    case FFSPLIT_E_UNSUPPORTED: return "combination not supported";
    case FFSPLIT_E_NONFINITE: return "NaN among the scores";
    case FFSPLIT_E_HIP: return "HIP runtime error";
    case FFSPLIT_E_TOO_LARGE: return "size beyond the fixed scratch of the entry point that allocates nothing";
    default: return "unknown status";
  }
}

size_t ffsplit_split_bytes(const ffsplit_desc_t* d) {
  if (check_desc(d, true) != FFSPLIT_OK) return 0;
  return make_layout(*d).total_bytes;
}

size_t ffsplit_workspace_bytes(const ffsplit_desc_t* d, int32_t call_id, int64_t T) {
  if (call_id == FFSPLIT_WS_SELECT) return d ? select_workspace_bytes(d->d_ff) : 0;
  if (check_desc(d, call_id != FFSPLIT_WS_SCORE) != FFSPLIT_OK || T < 0) return 0;
  const size_t esz = d->dtype == FFSPLIT_BF16 ? 2 : 4;
  if (call_id == FFSPLIT_WS_SCORE) {
    const ScoreWs w = make_score_ws(*d, T);
    return w.total_bytes;
  }
  if (call_id == FFSPLIT_WS_BUILD) return build_ws_bytes(*d);
  if (call_id == FFSPLIT_WS_FACTORIZE) {
    if (d->rem_kind != FFSPLIT_REM_LOWRANK) return 0;
    return build_ws_bytes(*d) + factorize_ws_bytes(*d);
  }
  if (call_id == FFSPLIT_WS_STACK) {
    const size_t fwd = ffsplit_workspace_bytes(d, FFSPLIT_WS_FORWARD, T);
    return fwd ? align256((size_t)T * d->d_model * esz) + fwd : 0;
  }
  if (call_id == FFSPLIT_WS_FORWARD) {
    const Layout L = make_layout(*d);
    const FwdWs w = make_fwd_ws(*d, L, T);
    (void)esz;
    return w.total_bytes;
  }
  return 0;
}

int ffsplit_score_neurons(const ffsplit_desc_t* d, const void* X, int64_t T, const void* W1, const void* Wg,
                          const void* W2, float* acc, int64_t* T_total, float* scores, int32_t score_kind,
                          void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_desc(d, false);
  if (rc) return rc;
  if (T < 0 || T > 0x7fffffff) return FFSPLIT_E_BADSHAPE;
  // The re-tiled (neuron-major) copy of the up projection lives at the start of the workspace;
  // a later batch of the same calibration run may reuse it instead of transposing again.
  const bool reuse_tiled = (score_kind & FFSPLIT_SCORE_REUSE_TILED) != 0;
  score_kind &= ~FFSPLIT_SCORE_REUSE_TILED;
  if (score_kind < 0 || score_kind > 2) return FFSPLIT_E_BADDESC;
  const bool glu = d->act == FFSPLIT_ACT_SWIGLU;
  if (!acc || !T_total || !W1 || (glu && !Wg) || (T > 0 && !X)) return FFSPLIT_E_NULLPTR;
  if (scores && score_kind != FFSPLIT_SCORE_ACT_ONLY && !W2) return FFSPLIT_E_NULLPTR;
  if (misaligned(X) || misaligned(W1) || misaligned(Wg) || misaligned(W2) || misaligned(acc) || misaligned(scores))
    return FFSPLIT_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const int bf16 = d->dtype == FFSPLIT_BF16;
  const int esz = bf16 ? 2 : 4;
  if (T > 0) {
    const ScoreWs w = make_score_ws(*d, T);
    if (!workspace || workspace_bytes < w.total_bytes) return FFSPLIT_E_WORKSPACE;
    if (((uintptr_t)workspace & 255u) != 0) return FFSPLIT_E_ALIGN;
    char* ws = (char*)workspace;
    void* Wt = ws + w.off_wt;
    float* p2 = (float*)(ws + w.off_p2);
    float* p1 = (float*)(ws + w.off_p1);
    // transposed (neuron-major) copy of the up projection(s); rows beyond d_ff are zero
    if (!reuse_tiled) FFS_TRY(launch_fill_zero(Wt, w.wt_bytes, st));
    PermArgs pa = {};
    pa.lds = d->d_ff;
    pa.dst = Wt;
    pa.ldd = w.dk;
    pa.dst_tiled = bf16;
    pa.n_count = d->d_ff;
    pa.c_count = d->d_model;
    if (reuse_tiled) {
      // nothing to do: the copy is in place
    } else if (glu) {
      pa.src = Wg; pa.glu_mode = 1;
      FFS_TRY(launch_permute_transpose(pa, esz, st));
      pa.src = W1; pa.glu_mode = 2;
      FFS_TRY(launch_permute_transpose(pa, esz, st));
    } else {
      pa.src = W1; pa.glu_mode = 0;
      FFS_TRY(launch_permute_transpose(pa, esz, st));
    }
    GemmArgs g = {};
    g.A = X; g.lda = d->d_model;
    g.Bt = Wt; g.ldb = w.dk;
    g.M = (int)T; g.N = w.n_gemm; g.K = d->d_model;
    g.group_m = 8;
    g.act_cols = w.n_gemm;
    g.part_s2 = p2; g.part_s1 = p1; g.n_out = w.n_out;
    if (bf16) FFS_TRY(launch_gemm_bf16(g, act_of(d), true, GEMM_256x128, 1, st));
    else FFS_TRY(launch_gemm_f32(g, act_of(d), true, st));
    FFS_TRY(launch_reduce_partials(p2, p1, w.tiles_m, w.n_out, d->d_ff, acc, st));
    *T_total += T;
  }
  if (scores)
    FFS_TRY(launch_finalize_scores(W2, bf16, d->d_model, d->d_ff, acc, (float)*T_total, score_kind, scores, st));
  return FFSPLIT_OK;
}

int ffsplit_select_heavy(const float* scores, int32_t d_ff, int32_t k, int32_t* idx, int32_t* perm,
                         int32_t* nan_flag, void* workspace, size_t workspace_bytes, void* stream) {
  if (d_ff <= 0) return FFSPLIT_E_BADDESC;
  if (k < 0 || k > d_ff) return FFSPLIT_E_BADSHAPE;
  if (!scores || (k > 0 && !idx)) return FFSPLIT_E_NULLPTR;
  if (!workspace || workspace_bytes < select_workspace_bytes(d_ff)) return FFSPLIT_E_WORKSPACE;
  if (misaligned(scores) || misaligned(workspace)) return FFSPLIT_E_ALIGN;
  FFS_TRY(launch_select(scores, d_ff, k, idx, perm, nan_flag, workspace, (hipStream_t)stream));
  return FFSPLIT_OK;
}

int ffsplit_select_heavy_static(const float* scores, int32_t d_ff, int32_t k, int32_t* idx, int32_t* perm,
                                int32_t* nan_flag, void* stream) {
  if (d_ff <= 0) return FFSPLIT_E_BADDESC;
  if (k < 0 || k > d_ff) return FFSPLIT_E_BADSHAPE;
  if (d_ff > select_static_max_dff()) return FFSPLIT_E_TOO_LARGE;
  if (!scores || (k > 0 && !idx)) return FFSPLIT_E_NULLPTR;
  if (misaligned(scores)) return FFSPLIT_E_ALIGN;
  FFS_TRY(launch_select_static(scores, d_ff, k, idx, perm, nan_flag, (hipStream_t)stream));
  return FFSPLIT_OK;
}

int ffsplit_build_split(const ffsplit_desc_t* d, const void* W1, const void* Wg, const void* W2,
                        const int32_t* idx, const void* const* factors, void* split, void* workspace,
                        size_t workspace_bytes, void* stream) {
  int rc = check_desc(d, true);
  if (rc) return rc;
  const bool glu = d->act == FFSPLIT_ACT_SWIGLU;
  const int k = d->k, m = d->d_ff - d->k, dm = d->d_model;
  if (!split || !W1 || !W2 || (glu && !Wg) || (k > 0 && !idx)) return FFSPLIT_E_NULLPTR;
  const bool lowrank = d->rem_kind == FFSPLIT_REM_LOWRANK && m > 0;
  if (lowrank) {
    if (!factors) return FFSPLIT_E_NULLPTR;
    for (int i = 0; i < 6; ++i) {
      const bool gate = (i == 2 || i == 3);
      if ((!gate || glu) && !factors[i]) return FFSPLIT_E_NULLPTR;
      if (misaligned(factors[i])) return FFSPLIT_E_ALIGN;
    }
  }
  if (misaligned(W1) || misaligned(Wg) || misaligned(W2) || ((uintptr_t)split & 255u)) return FFSPLIT_E_ALIGN;
  const bool need_rest = (d->rem_kind == FFSPLIT_REM_DENSE || d->rem_kind == FFSPLIT_REM_INT4 ||
                          d->rem_kind == FFSPLIT_REM_W3H8) && m > 0;
  const size_t ws_need = need_rest ? build_ws_bytes(*d) : 0;
  if (need_rest && (!workspace || workspace_bytes < ws_need)) return FFSPLIT_E_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int esz = d->dtype == FFSPLIT_BF16 ? 2 : 4;
  const Layout L = make_layout(*d);
  char* sp = (char*)split;
  FFS_TRY(launch_fill_zero(split, L.total_bytes, st));

  // remainder neurons in ascending order (needed when the library itself gathers them)
  int32_t* rest = nullptr;
  if (need_rest) {
    rest = (int32_t*)workspace;
    FFS_TRY(launch_rest_order(idx, k, d->d_ff, rest, (int32_t*)workspace + d->d_ff, st));
  }

  if (d->rem_kind == FFSPLIT_REM_INT4) {
    FFS_TRY(launch_int4_pack(*d, L, W1, Wg, W2, rest, idx, sp, st));
    return FFSPLIT_OK;
  }
  if (d->rem_kind == FFSPLIT_REM_W3H8) {
    FFS_TRY(launch_w3h8_pack(*d, L, W1, Wg, W2, rest, idx, sp, st));
    return FFSPLIT_OK;
  }

  // ---- heavy block: W1h^T (and Wgh^T) rows of B1t, W2h^T columns of B4t
  PermArgs pa = {};
  if (k > 0) {
    pa = {};
    pa.lds = d->d_ff; pa.dst = sp + L.off_b1; pa.ldd = L.dk; pa.dst_tiled = L.tiled;
    pa.n_count = k; pa.c_count = dm; pa.nmap = idx;
    if (glu) {
      pa.src = Wg; pa.glu_mode = 1; FFS_TRY(launch_permute_transpose(pa, esz, st));
      pa.src = W1; pa.glu_mode = 2; FFS_TRY(launch_permute_transpose(pa, esz, st));
    } else {
      pa.src = W1; pa.glu_mode = 0; FFS_TRY(launch_permute_transpose(pa, esz, st));
    }
    pa = {};
    pa.src = W2; pa.lds = dm; pa.dst = sp + L.off_b4; pa.ldd = L.k4; pa.dst_tiled = L.tiled;
    pa.n_count = dm; pa.c_count = k; pa.cmap = idx;
    FFS_TRY(launch_permute_transpose(pa, esz, st));
  }
  if (m == 0 || d->rem_kind == FFSPLIT_REM_NONE) return FFSPLIT_OK;

  if (d->rem_kind == FFSPLIT_REM_DENSE) {
    // remainder neurons appended to the same blocks after the padded heavy part
    pa = {};
    pa.lds = d->d_ff; pa.dst = sp + L.off_b1; pa.ldd = L.dk; pa.dst_tiled = L.tiled;
    pa.n_count = m; pa.c_count = dm; pa.nmap = rest;
    pa.row_off = (int64_t)L.n_up * L.kp;
    if (glu) {
      pa.src = Wg; pa.glu_mode = 1; FFS_TRY(launch_permute_transpose(pa, esz, st));
      pa.src = W1; pa.glu_mode = 2; FFS_TRY(launch_permute_transpose(pa, esz, st));
    } else {
      pa.src = W1; pa.glu_mode = 0; FFS_TRY(launch_permute_transpose(pa, esz, st));
    }
    pa = {};
    pa.src = W2; pa.lds = dm; pa.dst = sp + L.off_b4; pa.ldd = L.k4; pa.dst_tiled = L.tiled;
    pa.n_count = dm; pa.c_count = m; pa.cmap = rest; pa.coff = L.kp;
    FFS_TRY(launch_permute_transpose(pa, esz, st));
    return FFSPLIT_OK;
  }

  if (d->rem_kind == FFSPLIT_REM_LOWRANK) {
    const int r = d->rank;
    const void* P1 = factors[0]; const void* Q1 = factors[1];
    const void* Pg = factors[2]; const void* Qg = factors[3];
    const void* P2 = factors[4]; const void* Q2 = factors[5];
    // P^T rows of B1t after the heavy rows: [Pg^T ; P1^T] (SwiGLU) or [P1^T]
    pa = {};
    pa.lds = r; pa.dst = sp + L.off_b1; pa.ldd = L.dk; pa.dst_tiled = L.tiled; pa.n_count = r; pa.c_count = dm;
    pa.row_off = (int64_t)L.n_up * L.kp;
    if (glu) {
      pa.src = Pg; FFS_TRY(launch_permute_transpose(pa, esz, st));
      pa.row_off += L.rp;
    }
    pa.src = P1; FFS_TRY(launch_permute_transpose(pa, esz, st));
    // Q1^T (and Qg^T, interleaved in 32-row blocks): [n_up*mp, rp]
    pa = {};
    pa.lds = m; pa.dst = sp + L.off_q1; pa.ldd = L.rp; pa.dst_tiled = L.tiled; pa.n_count = m; pa.c_count = r;
    if (glu) {
      pa.src = Qg; pa.glu_mode = 1; FFS_TRY(launch_permute_transpose(pa, esz, st));
      pa.src = Q1; pa.glu_mode = 2; FFS_TRY(launch_permute_transpose(pa, esz, st));
    } else {
      pa.src = Q1; FFS_TRY(launch_permute_transpose(pa, esz, st));
    }
    // P2^T: [rp, mp]
    pa = {};
    pa.src = P2; pa.lds = r; pa.dst = sp + L.off_p2; pa.ldd = L.mp; pa.dst_tiled = L.tiled; pa.n_count = r; pa.c_count = m;
    FFS_TRY(launch_permute_transpose(pa, esz, st));
    // Q2^T into the columns of B4t after the heavy ones
    pa = {};
    pa.src = Q2; pa.lds = dm; pa.dst = sp + L.off_b4; pa.ldd = L.k4; pa.dst_tiled = L.tiled; pa.n_count = dm; pa.c_count = r;
    pa.coff = L.kp;
    FFS_TRY(launch_permute_transpose(pa, esz, st));
    return FFSPLIT_OK;
  }
  return FFSPLIT_E_UNSUPPORTED;
}

int ffsplit_factorize_remainder(const ffsplit_desc_t* d, const void* W1, const void* Wg, const void* W2,
                                const int32_t* idx, uint32_t seed, void* const* factors, void* workspace,
                                size_t workspace_bytes, void* stream) {
  int rc = check_desc(d, true);
  if (rc) return rc;
  if (d->rem_kind != FFSPLIT_REM_LOWRANK) return FFSPLIT_E_BADDESC;
  const bool glu = d->act == FFSPLIT_ACT_SWIGLU;
  const int m = d->d_ff - d->k;
  if (m <= 0) return FFSPLIT_OK;
  if (!W1 || !W2 || (glu && !Wg) || (d->k > 0 && !idx) || !factors) return FFSPLIT_E_NULLPTR;
  for (int i = 0; i < 6; ++i) {
    const bool gate = (i == 2 || i == 3);
    if ((!gate || glu) && !factors[i]) return FFSPLIT_E_NULLPTR;
    if (misaligned(factors[i])) return FFSPLIT_E_ALIGN;
  }
  if (misaligned(W1) || misaligned(Wg) || misaligned(W2)) return FFSPLIT_E_ALIGN;
  const size_t pre = build_ws_bytes(*d);
  if (!workspace || workspace_bytes < pre + factorize_ws_bytes(*d)) return FFSPLIT_E_WORKSPACE;
  if ((uintptr_t)workspace & 255u) return FFSPLIT_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  int32_t* rest = (int32_t*)workspace;
  FFS_TRY(launch_rest_order(idx, d->k, d->d_ff, rest, (int32_t*)workspace + d->d_ff, st));
  FFS_TRY(launch_factorize(*d, W1, Wg, W2, rest, seed, factors, (char*)workspace + pre, st));
  return FFSPLIT_OK;
}

static int forward_impl(const ffsplit_desc_t* d, const void* split, const void* X, int64_t T, void* Y, void* Y_heavy,
                        void* Y_rem, const ffsplit_epilogue_t* epi, void* workspace, size_t workspace_bytes,
                        void* stream) {
  int rc = check_desc(d, true);
  if (rc) return rc;
  if (T < 0 || T > 0x7fffffff) return FFSPLIT_E_BADSHAPE;
  if (T == 0) return FFSPLIT_OK;
  if (!split || !X || !Y) return FFSPLIT_E_NULLPTR;
  if (misaligned(X) || misaligned(Y) || misaligned(Y_heavy) || misaligned(Y_rem) || ((uintptr_t)split & 255u))
    return FFSPLIT_E_ALIGN;
  Epilogue ep = {};
  if (epi) {
    if (misaligned(epi->b1_packed) || misaligned(epi->b2) || misaligned(epi->residual)) return FFSPLIT_E_ALIGN;
    ep.b1 = epi->b1_packed; ep.b2 = epi->b2; ep.resid = epi->residual; ep.out_f32 = epi->y_f32 != 0;
    // a neuron's bias enters before the activation: built for the GeLU layers with bf16 / fp32
    // weights (the gated layers of the Llama family carry no biases)
    if (ep.b1 && (d->act != FFSPLIT_ACT_GELU || d->rem_kind == FFSPLIT_REM_INT4 || d->rem_kind == FFSPLIT_REM_W3H8))
      return FFSPLIT_E_UNSUPPORTED;
  }
  const Layout L = make_layout(*d);
  const FwdWs w = make_fwd_ws(*d, L, T);
  if (!workspace || workspace_bytes < w.total_bytes) return FFSPLIT_E_WORKSPACE;
  if ((uintptr_t)workspace & 255u) return FFSPLIT_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const char* sp = (const char*)split;
  char* ws = (char*)workspace;
  const int M = (int)T;
  const size_t ysz = ep.out_f32 ? 4 : 2;   // (quantised kinds are bf16)
  if (d->rem_kind == FFSPLIT_REM_W3H8) {
    if (M <= W3H8_DECODE_MAX_T) {
      // passes of at most 32 tokens, each streaming the packed codes once
      for (int t0 = 0; t0 < M; t0 += 32) {
        const size_t o = (size_t)t0 * d->d_model * 2;
        Epilogue e2 = ep;
        if (e2.resid) e2.resid += (size_t)t0 * d->d_model;
        const int r3 = w3h8_forward_small(*d, L, w, sp, (const char*)X + o, M - t0 < 32 ? M - t0 : 32,
                                          (char*)Y + (size_t)t0 * d->d_model * ysz,
                                          Y_heavy ? (char*)Y_heavy + o : nullptr, Y_rem ? (char*)Y_rem + o : nullptr, e2,
                                          ws, st);
        if (r3) return r3 == -2 ? FFSPLIT_E_UNSUPPORTED : FFSPLIT_E_HIP;
      }
      return FFSPLIT_OK;
    }
    ffsplit_desc_t dd = *d;
    dd.rem_kind = FFSPLIT_REM_DENSE;
    const Layout LD = make_layout(dd);
    const FwdWs wd = make_fwd_ws(dd, LD, T);
    FFS_TRY(launch_w3h8_expand(*d, L, LD, sp, ws + w.off_img, st));
    return forward_chain(&dd, LD, wd, ws + w.off_img, X, M, Y, Y_heavy, Y_rem, ep, ws + w.off_dense, st);
  }
  if (d->rem_kind == FFSPLIT_REM_INT4) {
    if (w.i4_prefill) {
      // many tokens: expand the int4 remainder to bf16 once, then the dense chain on MFMA tiles
      ffsplit_desc_t dd = *d;
      dd.rem_kind = FFSPLIT_REM_DENSE;
      const Layout LD = make_layout(dd);
      const FwdWs wd = make_fwd_ws(dd, LD, T);
      FFS_TRY(launch_int4_expand(*d, L, LD, sp, ws + w.off_img, st));
      return forward_chain(&dd, LD, wd, ws + w.off_img, X, M, Y, Y_heavy, Y_rem, ep, ws + w.off_dense, st);
    }
    const int r4 = int4_forward(*d, L, w, sp, X, M, Y, Y_heavy, Y_rem, ep, ws, st);
    return r4 == 0 ? FFSPLIT_OK : (r4 == -2 ? FFSPLIT_E_UNSUPPORTED : FFSPLIT_E_HIP);
  }
  return forward_chain(d, L, w, sp, X, M, Y, Y_heavy, Y_rem, ep, ws, st);
}

int ffsplit_forward(const ffsplit_desc_t* d, const void* split, const void* X, int64_t T, void* Y, void* Y_heavy,
                    void* Y_rem, void* workspace, size_t workspace_bytes, void* stream) {
  return forward_impl(d, split, X, T, Y, Y_heavy, Y_rem, nullptr, workspace, workspace_bytes, stream);
}

int ffsplit_forward_ex(const ffsplit_desc_t* d, const void* split, const void* X, int64_t T, void* Y, void* Y_heavy,
                       void* Y_rem, const ffsplit_epilogue_t* epilogue, void* workspace, size_t workspace_bytes,
                       void* stream) {
  return forward_impl(d, split, X, T, Y, Y_heavy, Y_rem, epilogue, workspace, workspace_bytes, stream);
}

size_t ffsplit_neuron_bias_floats(const ffsplit_desc_t* d) {
  if (check_desc(d, true) != FFSPLIT_OK) return 0;
  return (size_t)round_up(d->k, 64) + (size_t)round_up(d->d_ff - d->k, 64);
}

int ffsplit_pack_neuron_bias(const ffsplit_desc_t* d, const void* b1, const int32_t* idx, float* b1_packed,
                             void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_desc(d, true);
  if (rc) return rc;
  if (!b1 || !b1_packed || (d->k > 0 && !idx)) return FFSPLIT_E_NULLPTR;
  if (misaligned(b1) || misaligned(b1_packed)) return FFSPLIT_E_ALIGN;
  if (!workspace || workspace_bytes < build_ws_bytes(*d)) return FFSPLIT_E_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  int32_t* rest = (int32_t*)workspace;
  FFS_TRY(launch_rest_order(idx, d->k, d->d_ff, rest, (int32_t*)workspace + d->d_ff, st));
  FFS_TRY(launch_pack_neuron_bias(b1, d->dtype == FFSPLIT_BF16, idx, rest, d->k, round_up(d->k, 64), d->d_ff - d->k,
                                  round_up(d->d_ff - d->k, 64), b1_packed, st));
  return FFSPLIT_OK;
}

int ffsplit_token_rmsnorm(const float* x, int64_t T, int32_t d_model, float eps, int32_t dtype, void* out,
                          void* stream) {
  if (d_model <= 0 || d_model % 8 != 0 || T < 0 || T > 0x7fffffff) return FFSPLIT_E_BADSHAPE;
  if (dtype != FFSPLIT_F32 && dtype != FFSPLIT_BF16) return FFSPLIT_E_BADDESC;
  if (T == 0) return FFSPLIT_OK;
  if (!x || !out) return FFSPLIT_E_NULLPTR;
  if (misaligned(x) || misaligned(out)) return FFSPLIT_E_ALIGN;
  FFS_TRY(launch_token_rmsnorm(x, T, d_model, eps, dtype == FFSPLIT_BF16, out, (hipStream_t)stream));
  return FFSPLIT_OK;
}

int ffsplit_stack_forward(const ffsplit_desc_t* d, int32_t n_layers, const void* const* splits,
                          const float* const* b1_packed, const float* const* b2, float* x, int64_t T, float eps,
                          void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_desc(d, true);
  if (rc) return rc;
  if (n_layers < 0 || T < 0 || T > 0x7fffffff) return FFSPLIT_E_BADSHAPE;
  if (n_layers == 0 || T == 0) return FFSPLIT_OK;
  if (!splits || !x) return FFSPLIT_E_NULLPTR;
  for (int l = 0; l < n_layers; ++l)
    if (!splits[l]) return FFSPLIT_E_NULLPTR;
  if (misaligned(x)) return FFSPLIT_E_ALIGN;
  const size_t esz = d->dtype == FFSPLIT_BF16 ? 2 : 4;
  const size_t xn_bytes = align256((size_t)T * d->d_model * esz);
  const size_t fwd = ffsplit_workspace_bytes(d, FFSPLIT_WS_FORWARD, T);
  if (!workspace || workspace_bytes < xn_bytes + fwd) return FFSPLIT_E_WORKSPACE;
  if ((uintptr_t)workspace & 255u) return FFSPLIT_E_ALIGN;
  char* xn = (char*)workspace;
  for (int l = 0; l < n_layers; ++l) {
    // x <- x + FFN_l(n(x)): the normalised tokens in the storage type, the sum back into the fp32 stream
    rc = ffsplit_token_rmsnorm(x, T, d->d_model, eps, d->dtype, xn, stream);
    if (rc) return rc;
    ffsplit_epilogue_t e = {};
    e.b1_packed = b1_packed ? b1_packed[l] : nullptr;
    e.b2 = b2 ? b2[l] : nullptr;
    e.residual = x;
    e.y_f32 = 1;
    rc = forward_impl(d, splits[l], xn, T, x, nullptr, nullptr, &e, xn + xn_bytes, workspace_bytes - xn_bytes, stream);
    if (rc) return rc;
  }
  return FFSPLIT_OK;
}

int ffsplit_split_export(const ffsplit_desc_t* d, const void* split, int32_t what, int8_t* q_out, uint16_t* s_out,
                         void* stream) {
  int rc = check_desc(d, true);
  if (rc) return rc;
  if (d->rem_kind != FFSPLIT_REM_INT4 && d->rem_kind != FFSPLIT_REM_W3H8) return FFSPLIT_E_UNSUPPORTED;
  if (!split || !q_out || !s_out) return FFSPLIT_E_NULLPTR;
  const int what_max = d->rem_kind == FFSPLIT_REM_W3H8 ? 5 : 2;
  if (what < 0 || what > what_max || (what % 3 == 1 && d->act != FFSPLIT_ACT_SWIGLU)) return FFSPLIT_E_BADDESC;
  const Layout L = make_layout(*d);
  if (d->rem_kind == FFSPLIT_REM_W3H8) {
    FFS_TRY(launch_w3h8_export(*d, L, (const char*)split, what, q_out, s_out, (hipStream_t)stream));
    return FFSPLIT_OK;
  }
  FFS_TRY(launch_int4_export(*d, L, (const char*)split, what, q_out, s_out, (hipStream_t)stream));
  return FFSPLIT_OK;
}

}  // extern "C"
