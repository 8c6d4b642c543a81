/*
 * libffsplit: the split feed-forward layer of FFSplit (arXiv 2401.04044) on
 * one AMD MI355X (gfx950).
 *
 * The feed-forward layer FFN(X) = sigma(X U) V is a sum of d_ff rank-one terms,
 * one per neuron (Sec. 2, Eq. 1).  Neurons are scored on a calibration token
 * set (Sec. 4.1, Eq. 3), the k highest-scoring ones form the heavy set h2, and
 * the layer is evaluated as FFN_1 (heavy neurons, weights untouched) plus FFN_2
 * (the remaining neurons, compressed) (Sec. 2, Eq. 2; Sec. 4.2).
 *
 * Names: W1 = up projection (the paper's U, [d_model, d_ff]); Wg = SwiGLU gate
 * ([d_model, d_ff]); W2 = down projection (the paper's V, [d_ff, d_model]).
 * A neuron is one column of W1 (and Wg) together with the matching row of W2.
 *
 * Conventions for every call
 *   - Every pointer is a DEVICE pointer unless its comment says "host".
 *   - Matrices are row-major and contiguous; device pointers are 16-byte aligned.
 *   - Element type of X, Y and all dense weights/factors is desc->dtype.
 *   - The library allocates nothing, keeps no state between calls (apart from
 *     a set-once, thread-safe note per device that a kernel's shared-memory limit
 *     has been raised, or that the device refused it and the kernel is not used there)
 *     and never synchronises: a call validates its arguments on the host, enqueues
 *     kernels on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and returns.  Outputs are valid once the caller has synchronised the stream.
 *   - Caller owns every buffer.  `workspace` is scratch of at least
 *     ffsplit_workspace_bytes(...) bytes, 256-byte aligned, contents undefined
 *     on entry and on exit; it may be reused by later calls on the same stream.
 *   - Return value: FFSPLIT_OK or a negative FFSPLIT_E_* code.  Argument errors
 *     are found before anything is launched.
 *   - T = 0, k = 0 and k = d_ff are valid (the empty part contributes zero).
 *   - Results are deterministic: the same call on the same inputs gives the
 *     same bits (no floating-point atomics anywhere).
 */
#ifndef FFSPLIT_H
#define FFSPLIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { FFSPLIT_ACT_GELU = 0,      /* GeLU z*Phi(z) (the erf form, not the tanh fit)       */
       FFSPLIT_ACT_SWIGLU = 1 };  /* silu(X Wg) * (X W1)                                  */
/* How the activation is evaluated.  F32: erff / expf.  BF16 (the forward pass at any
 * batch size with dense or low-rank or W3H8 parts, and the calibration pass):
 * Phi(-|z|) = 2^q(|z|) with q a cubic fitted to log2 Phi (max absolute error of
 * z*Phi(z) 5.7e-5, relative error up to 0.25 % for |z| < 0.03: at most one bf16 unit
 * in the last place of the result, which is stored in bf16), silu through exp2 and a
 * reciprocal.  The int4 small-batch kernels: erff / expf.  The calibration pass ranks
 * what the forward pass computes.                                                  */
enum { FFSPLIT_F32 = 0, FFSPLIT_BF16 = 1 };
enum { FFSPLIT_REM_NONE = 0,      /* FFN_2 dropped                                        */
       FFSPLIT_REM_DENSE = 1,     /* FFN_2 kept uncompressed                              */
       FFSPLIT_REM_LOWRANK = 2,   /* each remainder matrix given as two rank-r factors    */
       FFSPLIT_REM_INT4 = 3,      /* remainder weights as group-wise symmetric int4       */
       FFSPLIT_REM_W3H8 = 4 };    /* heavy weights int8, remainder int3, both group-wise  */
enum { FFSPLIT_SCORE_SUMSQ = 0,   /* Eq. 3: ||sigma(X U[:,j])||_F^2 * ||V[j,:]||_F^2      */
       FFSPLIT_SCORE_MEAN_L2 = 1, /* mean_t ||sigma(x_t U[:,j]) V[j,:]||_2                */
       FFSPLIT_SCORE_ACT_ONLY = 2 /* ||sigma(X U[:,j])||_F^2 (Sec. 2's heavy-hitter norm) */ };
/* Flag, or-ed into score_kind: this batch continues a calibration run on the same desc, the
 * same W1 / Wg and the same workspace as the previous ffsplit_score_neurons call, whose
 * re-tiled copy of the up projection (the first bytes of the workspace, independent of T as
 * long as the workspace was sized for the largest batch) is reused instead of being rebuilt.
 * The caller must not have used the workspace for anything else in between.            */
#define FFSPLIT_SCORE_REUSE_TILED 0x100
enum { FFSPLIT_WS_SCORE = 0, FFSPLIT_WS_SELECT = 1, FFSPLIT_WS_BUILD = 2, FFSPLIT_WS_FORWARD = 3,
       FFSPLIT_WS_FACTORIZE = 4, FFSPLIT_WS_STACK = 5 };

enum { FFSPLIT_OK = 0,
       FFSPLIT_E_NULLPTR = -1,     /* a required pointer is NULL                          */
       FFSPLIT_E_BADDESC = -2,     /* unknown act / dtype / rem_kind, non-positive sizes  */
       FFSPLIT_E_BADSHAPE = -3,    /* k > d_ff, rank > min(d_model, m), group does not    */
                                   /* divide d_model, d_model % 8 != 0, T < 0             */
       FFSPLIT_E_ALIGN = -4,       /* a pointer is not 16-byte aligned                    */
       FFSPLIT_E_WORKSPACE = -5,   /* workspace missing or too small                      */
       FFSPLIT_E_UNSUPPORTED = -6, /* valid but not implemented combination               */
       FFSPLIT_E_NONFINITE = -7,   /* reported through select_heavy's device flag only    */
       FFSPLIT_E_HIP = -8,         /* a HIP runtime call failed                           */
       FFSPLIT_E_TOO_LARGE = -9    /* beyond the fixed scratch of a *_static entry point  */ };

/* Plain data, passed by pointer, never retained. */
typedef struct {
  int32_t d_model;   /* d; multiple of 8                                                  */
  int32_t d_ff;      /* number of neurons                                                 */
  int32_t act;       /* FFSPLIT_ACT_*                                                     */
  int32_t dtype;     /* FFSPLIT_F32 / FFSPLIT_BF16                                        */
  int32_t k;         /* |h2|, 0..d_ff                                                     */
  int32_t rem_kind;  /* FFSPLIT_REM_*                                                     */
  int32_t rank;      /* LOWRANK: r, the same for every factored matrix                    */
  int32_t group;     /* INT4, W3H8: group length along d_model (must divide it; multiple of 32) */
} ffsplit_desc_t;

/* Static description of a status code. */
const char* ffsplit_status_string(int status);

/* Bytes of scratch the given call needs for T tokens (pure host arithmetic). */
size_t ffsplit_workspace_bytes(const ffsplit_desc_t* desc, int32_t call_id, int64_t T);

/* Bytes of the packed split produced by ffsplit_build_split (pure host arithmetic). */
size_t ffsplit_split_bytes(const ffsplit_desc_t* desc);

/*
 * Calibration, one token batch (Sec. 4.2 first step; Sec. 4.1, Eq. 3).
 * For every neuron j adds this batch to the running sums
 *     acc[j]        += sum_t H[t,j]^2        acc[d_ff + j] += sum_t |H[t,j]|
 * with H = gelu(X W1) or silu(X Wg) * (X W1), computed on the unmodified dense
 * weights, and adds T to *T_total.  If `scores` is not NULL it then writes
 *     SUMSQ    scores[j] = acc[j] * sum_c W2[j,c]^2
 *     MEAN_L2  scores[j] = acc[d_ff+j] / T_total * sqrt(sum_c W2[j,c]^2)
 *     ACT_ONLY scores[j] = acc[j]
 * X [T, d_model]; W1, Wg [d_model, d_ff]; W2 [d_ff, d_model] (Wg NULL unless
 * SWIGLU; W2 may be NULL when scores is NULL).  acc: [2*d_ff] fp32, owned and
 * zeroed by the caller before the first batch (calibration can be resumed by
 * keeping acc and *T_total).  T_total: host pointer, in/out.  scores: [d_ff] fp32.
 * desc->k, rem_kind, rank, group are ignored.
 */
int ffsplit_score_neurons(const ffsplit_desc_t* desc, const void* X, int64_t T,
                          const void* W1, const void* Wg, const void* W2,
                          float* acc, int64_t* T_total, float* scores, int32_t score_kind,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Heavy-hitter selection (Sec. 4.1 / 5.1.1: the neurons with the highest score).
 * Writes to idx[0..k) the indices of the k largest scores ordered by score
 * descending, equal scores by ascending index; -0 counts as +0, +Inf as the
 * largest value.  If perm is not NULL it receives the neuron permutation
 * [idx ; every other index ascending] of length d_ff (Eq. 2's partition).
 * If a score is NaN, *nan_flag (if not NULL) is set to FFSPLIT_E_NONFINITE,
 * else to 0; idx is then still a valid set of distinct indices (NaN ranks as
 * the largest value).  scores: [d_ff] fp32, all >= 0 or NaN.  Bit-exact.
 */
int ffsplit_select_heavy(const float* scores, int32_t d_ff, int32_t k,
                         int32_t* idx, int32_t* perm, int32_t* nan_flag,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * ffsplit_select_heavy for callers that cannot allocate or size a workspace:
 * code under HIP graph capture, tight serving loops that re-select per request,
 * harnesses that forbid hipMalloc.  Same results, same argument meaning; the
 * scratch is a fixed array inside the library (FFSPLIT_SELECT_STATIC_MAX_DFF * 12
 * + 256 bytes of device memory per GPU, held until the process ends), so
 *   - d_ff > FFSPLIT_SELECT_STATIC_MAX_DFF returns FFSPLIT_E_TOO_LARGE (nothing
 *     is launched);
 *   - the call allocates nothing and frees nothing (the first call on a device
 *     looks the array's address up once, with that device current);
 *   - every call on one GPU uses the same array: calls that overlap in time on
 *     one GPU (two streams, two threads) race.  Calls on one stream are safe.
 * Nothing in the array has to be cleared between calls.
 */
#define FFSPLIT_SELECT_STATIC_MAX_DFF 65536
int ffsplit_select_heavy_static(const float* scores, int32_t d_ff, int32_t k,
                                int32_t* idx, int32_t* perm, int32_t* nan_flag,
                                void* stream);

/*
 * Split construction (Eq. 2; Fig. 3: U1 = U[:,h2], V1 = V[h2,:], U2, V2 the
 * rest; Sec. 4.2: only U2, V2 are compressed).  Gathers the heavy neurons'
 * columns/rows into dense blocks and packs the remainder into `split`
 * (ffsplit_split_bytes(desc) bytes, 256-byte aligned; private layout,
 * position independent so it may be copied).
 *   idx      [k] distinct neuron indices (int32), any order.
 *   DENSE    remainder columns/rows gathered in ascending index order.
 *   LOWRANK  factors (HOST array of 6 device pointers P1, Q1, Pg, Qg, P2, Q2)
 *            with W1[:,rest] ~= P1 Q1, Wg[:,rest] ~= Pg Qg, W2[rest,:] ~= P2 Q2,
 *            rest = the non-heavy neurons ascending; P1, Pg [d_model, r];
 *            Q1, Qg [r, m]; P2 [m, r]; Q2 [r, d_model]; Pg, Qg NULL unless
 *            SWIGLU.  W1, Wg, W2 are read for the heavy part only.
 *   INT4     each remainder neuron's W1 column, Wg column and W2 row (all of
 *            length d_model) is quantised round-to-nearest in groups of
 *            desc->group (Sec. 5.2), in fp32:  a = max|w|, s = fp16(a / 7),
 *            q = s == 0 ? 0 : clamp(rint(w / float(s)), -8, 7) (ties to even),
 *            dequantised value float(s) * q.  Requires dtype BF16.
 *   W3H8     Sec. 5.2's setting for the LLMs: the same quantiser at 3 bits
 *            (a / 3, codes -4..3) on the remainder and at 8 bits (a / 127,
 *            codes -128..127) on the heavy neurons' columns and rows, which
 *            are therefore not kept in bf16.  Requires dtype BF16.
 */
int ffsplit_build_split(const ffsplit_desc_t* desc, const void* W1, const void* Wg,
                        const void* W2, const int32_t* idx, const void* const* factors,
                        void* split, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Rank-r factors of the remainder matrices, computed on the device, in the form
 * ffsplit_build_split takes for LOWRANK (Sec. 4.2 / 5.1.1: a low-rank
 * decomposition of U2 and V2, each matrix on its own).  In place of a full SVD
 * this is the randomised range finder of Halko, Martinsson and Tropp (2011,
 * Alg. 4.1) on the d_model side of each matrix: with Z [d_model, m] =
 * W1[:, rest], Wg[:, rest] or W2[rest, :]^T (rest = the non-heavy neurons
 * ascending), Y = Z Omega^T for a Rademacher test matrix Omega [r, m], B an
 * orthonormal basis of range(Y), the approximation is Z ~= B (B^T Z).
 *   P1 = B, Q1 = B^T Z (likewise Pg, Qg);  Q2 = B^T, P2 = Z^T B.
 * Omega(i, j) = +1 / -1 from the top bit of
 *   fmix32((i m + j) * 0x9E3779B1 + fmix32(seed + 0x9E3779B9 * stream)),
 * fmix32 = the 32-bit finaliser of MurmurHash3, stream = 0 (W1), 1 (Wg), 2 (W2):
 * the same signs on every machine.  All arithmetic in fp32; the factors are
 * written in desc->dtype.  Only their products are determined (the basis B is
 * fixed up to a rotation).  desc: rem_kind LOWRANK, 0 < rank <= min(d_model, m).
 * factors: HOST array of 6 device pointers P1 [d_model, r], Q1 [r, m], Pg, Qg,
 * P2 [m, r], Q2 [r, d_model] (Pg, Qg may be NULL unless SWIGLU), written.
 * workspace: ffsplit_workspace_bytes(desc, FFSPLIT_WS_FACTORIZE, 0).
 */
int ffsplit_factorize_remainder(const ffsplit_desc_t* desc, const void* W1, const void* Wg,
                                const void* W2, const int32_t* idx, uint32_t seed,
                                void* const* factors, void* workspace, size_t workspace_bytes,
                                void* stream);

/*
 * Split forward pass (Eq. 2):  Y = FFN_1(X) + FFN_2~(X), with
 * FFN_1 = act(X W1[:,h2] [, X Wg[:,h2]]) W2[h2,:] and FFN_2~ the remainder in
 * its compressed form (LOWRANK: act((X P1) Q1 [, (X Pg) Qg]) P2 Q2).
 * X [T, d_model]; Y [T, d_model].  Y_heavy / Y_rem: NULL, or [T, d_model]
 * buffers that receive FFN_1(X) and FFN_2~(X) separately (diagnostic; costs
 * extra launches).  Accumulation is fp32; intermediates between the chained
 * products are stored in desc->dtype.
 * LOWRANK: the activated remainder act((X P1) Q1) [T, m] is such an intermediate,
 * except for un-gated BF16 layers of rank 449..512 from 8192 tokens on, where it
 * is multiplied by P2 chunk by chunk without being stored (rounded to bf16 all
 * the same; only the order of the fp32 partial sums differs).
 * INT4: up to 192 tokens run in passes of 16 through weight-streaming kernels
 * that apply the group scales in fp32; above that the dequantised weights
 * float(s) * q are first written once, rounded to bf16, into the workspace
 * (which is why ffsplit_workspace_bytes grows with a dense copy of the layer
 * there) and the products run on them.
 * W3H8: up to 128 tokens run in passes of 32 that stream the packed codes
 * (scales applied in fp32 or fp16, the activations between the two products
 * kept in fp16, saturating); larger batches expand the weights to
 * bf16(float(s) * q) first as above.
 */
int ffsplit_forward(const ffsplit_desc_t* desc, const void* split, const void* X, int64_t T,
                    void* Y, void* Y_heavy, void* Y_rem,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * The layer as the models of Sec. 5.1 / 5.2 wrap it: biases and the residual
 * connection around the split feed-forward layer, fused into the products'
 * store steps (Sec. 2's first equation omits the biases that BERT and OPT have;
 * Sec. 4.1 applies the split "at each layer" of such a model).
 *   Y = [residual +] FFN_1(X) + FFN_2~(X) [+ b2],
 *   FFN_1 = gelu(X W1[:,h2] + b1[h2]) W2[h2,:], and the remainder's biases enter
 *   its compressed pre-activation: gelu((X P1) Q1 + b1[rest]) P2 Q2.
 * A neuron's bias belongs to the neuron and moves with it in Eq. 2's partition;
 * b2 is added once.  Every field may be NULL / 0:
 *   b1_packed  fp32 [ffsplit_neuron_bias_floats(desc)], from ffsplit_pack_neuron_bias.
 *              GELU with NONE / DENSE / LOWRANK only (else FFSPLIT_E_UNSUPPORTED).
 *   b2         fp32 [d_model].
 *   residual   fp32 [T, d_model]; may be the same buffer as Y when y_f32 is set
 *              (every element is read, then written, by one thread).
 *   y_f32      Y is float [T, d_model] instead of desc->dtype (the fp32 residual
 *              stream of a layer stack).  Y_heavy / Y_rem stay in desc->dtype and
 *              carry neither b2 nor the residual.
 * A layer with no neuron at all (k = 0 and no remainder) cannot carry an
 * epilogue: FFSPLIT_E_UNSUPPORTED.
 */
typedef struct {
  const float* b1_packed;
  const float* b2;
  const float* residual;
  int32_t y_f32;
} ffsplit_epilogue_t;

int ffsplit_forward_ex(const ffsplit_desc_t* desc, const void* split, const void* X, int64_t T,
                       void* Y, void* Y_heavy, void* Y_rem, const ffsplit_epilogue_t* epilogue,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Floats of a packed neuron-bias vector: round_up(k, 64) + round_up(d_ff - k, 64). */
size_t ffsplit_neuron_bias_floats(const ffsplit_desc_t* desc);

/*
 * b1 [d_ff] (desc->dtype, original neuron order) -> b1_packed in the packed
 * split's neuron order: b1[idx[0..k)], zeros up to round_up(k, 64), then b1 of
 * the other neurons ascending, zeros up to the end.  idx as given to
 * ffsplit_build_split.  workspace: ffsplit_workspace_bytes(desc, FFSPLIT_WS_BUILD, 0).
 */
int ffsplit_pack_neuron_bias(const ffsplit_desc_t* desc, const void* b1, const int32_t* idx,
                             float* b1_packed, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Per-token RMS normalisation n(x) = x / sqrt(mean(x^2) + eps), no learned
 * scale: the pre-norm of the layer stack below.  x fp32 [T, d_model];
 * out [T, d_model] in `dtype` (FFSPLIT_F32 / FFSPLIT_BF16).  d_model % 8 == 0.
 */
int ffsplit_token_rmsnorm(const float* x, int64_t T, int32_t d_model, float eps, int32_t dtype,
                          void* out, void* stream);

/*
 * A stack of n_layers split feed-forward layers of one shape on an fp32 residual
 * stream (Sec. 4.1: the split is applied at each layer; the 40-layer workload):
 *   for l in 0..n_layers:  x <- x + FFN_split_l(n(x)) [+ b2_l],
 * n = ffsplit_token_rmsnorm in desc->dtype, the addition fused into the last
 * product of each layer (ffsplit_forward_ex with residual = Y = x, y_f32 = 1).
 * splits: HOST array of n_layers device pointers (packed splits of `desc`);
 * b1_packed, b2: NULL or HOST arrays of n_layers device pointers (entries may
 * be NULL).  x [T, d_model] fp32, in place.
 * workspace: ffsplit_workspace_bytes(desc, FFSPLIT_WS_STACK, T).
 */
int ffsplit_stack_forward(const ffsplit_desc_t* desc, int32_t n_layers, const void* const* splits,
                          const float* const* b1_packed, const float* const* b2,
                          float* x, int64_t T, float eps,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measured ceilings of the machine, for the benchmark's report (nothing on the
 * path calls them; the throughput figures are quoted against the datasheet peaks
 * and, beside them, against these):
 *   ffsplit_probe_mfma         `workgroups` x 4 wavefronts each issue `iters` x 8
 *                              independent v_mfma_f32_32x32x16_bf16, no memory
 *                              traffic; *flops (host) receives the flop count.
 *   ffsplit_probe_stream_read  reads buf[0, bytes) once with 16-byte loads, eight in
 *                              flight per thread, from `workgroups` x 256 threads.
 * scratch: at least 16 bytes of device memory (never written in practice).
 */
int ffsplit_probe_mfma(int32_t workgroups, int32_t iters, void* scratch, double* flops, void* stream);
int ffsplit_probe_stream_read(const void* buf, size_t bytes, int32_t workgroups, void* scratch, void* stream);

/*
 * Test hook: unpack the quantised weights of a built split (INT4, W3H8) into
 * logical order.  what = 0 (W1 columns), 1 (Wg columns), 2 (W2 rows) of the
 * remainder: q_out [m, d_model] int8 codes, s_out [m, d_model/group] fp16 scale
 * bits (uint16), neuron order = remainder ascending.  W3H8 only: what = 3, 4, 5
 * likewise for the heavy neurons ([k, ...], in the order of idx).
 */
int ffsplit_split_export(const ffsplit_desc_t* desc, const void* split, int32_t what,
                         int8_t* q_out, uint16_t* s_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FFSPLIT_H */
