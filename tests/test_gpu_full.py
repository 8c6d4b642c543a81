"""Full-size runs of the five workloads in the launch configuration the benchmark
times.  Forward outputs are compared with the oracle on EVERY row (relative
Frobenius error and the worst row); only the 65 536-token run and the scores of
the large layers are checked on samples (rows of X and columns of W1 are
independent, so the oracle's result for a sample is exactly what the full run
must produce for it).  Heavy sets are compared in full (bit-exact as sets, and
the ranking kernel against the oracle's rule on the GPU's own scores)."""
import numpy as np
import pytest
import torch

from oracle import ffsplit_oracle as orc
import workloads as wl
from workloads.configs import C1, C2, C3, C4, C5
from gpu_util import (guarded_forward, TOL, dev, host, relf, assert_close, assert_scores_close, desc_for, layer_to_dev,
                      gpu_scores, Guarded)

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]


@pytest.fixture(scope="module")
def ff():
    import paper_2401_04044_amd as m
    return m


def calibrate_and_select(ff, cfg, L, Ld, n_batches=2):
    X = wl.make_tokens(cfg, cfg.calib_T, wl.gen.S_CALIB)
    step = (cfg.calib_T + n_batches - 1) // n_batches
    xs = [dev(X[i:i + step], cfg.dtype) for i in range(0, cfg.calib_T, step)]
    scores, acc, tt = gpu_scores(ff, desc_for(ff, cfg, "none"), Ld, xs)
    assert tt == cfg.calib_T
    idx, _, flag = ff.select_heavy(scores, cfg.k)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    assert int(flag.item()) == 0
    assert np.array_equal(idx_h, orc.select_heavy(scores.cpu().numpy(), cfg.k))     # ranking kernel, bit-exact
    assert np.array_equal(np.sort(idx_h), L["planted"])                              # the oracle's heavy set
    return X, scores, idx, idx_h


def sampled_rows(T, n, seed=0):
    if T <= n:
        return np.arange(T)
    rows = np.random.default_rng(seed).choice(T, n - 2, replace=False)
    return np.unique(np.concatenate([rows, [0, T - 1]]))


def test_c1_bert_shape_fp32_full(ff):
    cfg = C1
    L = wl.make_layer(cfg)
    Ld = layer_to_dev(L, cfg.dtype)
    Xc, scores, idx, idx_h = calibrate_and_select(ff, cfg, L, Ld, n_batches=1)
    acc_o = orc.score_accumulate(orc.new_accumulator(cfg.d_ff), Xc, L["W1"], None, "gelu")
    want_s = orc.neuron_scores(acc_o, L["W2"])
    assert_scores_close(scores.cpu().numpy(), want_s, "f32", "C1")
    assert np.array_equal(np.sort(idx_h), np.sort(orc.select_heavy(want_s, cfg.k)))
    fac = wl.make_factors(cfg, L, idx_h)
    desc = desc_for(ff, cfg)
    split = ff.build_split(desc, Ld["W1"], None, Ld["W2"], idx, {k: dev(v, "f32") for k, v in fac.items()})
    X = wl.make_tokens(cfg, cfg.prefill_T)
    Y, Yh, Yr = guarded_forward(ff, desc, split, dev(X, "f32"), want_parts=True)
    torch.cuda.synchronize()
    want = orc.forward_split(X, L["W1"], L["W2"], None, idx_h, "gelu", "lowrank", fac)
    for g, w, nm in zip((Y, Yh, Yr), want, ("Y", "Y_heavy", "Y_rem")):
        assert_close(host(g), w, "f32", f"C1 {nm}")


def test_c2_opt13b_shape_full_pipeline(ff):
    cfg = C2
    L = wl.make_layer(cfg)
    Ld = layer_to_dev(L, cfg.dtype)
    Xc, scores, idx, idx_h = calibrate_and_select(ff, cfg, L, Ld)
    # scores against the oracle on a sample of neurons (columns are independent)
    cols = np.concatenate([L["planted"][:16], np.random.default_rng(1).choice(cfg.d_ff, 48, replace=False)])
    acc_o = orc.score_accumulate(orc.new_accumulator(len(cols)), Xc, L["W1"][:, cols], None, "gelu")
    want_s = orc.neuron_scores(acc_o, L["W2"][cols, :])
    assert_scores_close(scores.cpu().numpy()[cols], want_s, "bf16", "C2 sampled neurons")
    fac = wl.make_factors(cfg, L, idx_h)
    desc = desc_for(ff, cfg)
    split = ff.build_split(desc, Ld["W1"], None, Ld["W2"], idx, {k: dev(v, "bf16") for k, v in fac.items()})
    T = cfg.prefill_T
    X = wl.make_tokens(cfg, T)
    Y, Yh, Yr = guarded_forward(ff, desc, split, dev(X, "bf16"), want_parts=True)
    Y2 = guarded_forward(ff, desc, split, dev(X, "bf16"))
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)                              # deterministic
    want = orc.forward_split(X, L["W1"], L["W2"], None, idx_h, "gelu", "lowrank", fac)      # all 4096 rows
    for g, w, nm in zip((Y, Yh, Yr), want, ("Y", "Y_heavy", "Y_rem")):
        assert_close(host(g), w, "bf16", f"C2 T={T} {nm}")


def test_c2_opt13b_shape_factorize_on_device(ff):
    """The rank-512 factors of the C2 remainder computed by the library itself: products
    against the oracle's, then build + forward on them (sampled rows)."""
    cfg = C2
    L = wl.make_layer(cfg)
    Ld = layer_to_dev(L, cfg.dtype)
    idx_h = L["planted"]
    idx = torch.from_numpy(idx_h).cuda()
    desc = desc_for(ff, cfg)
    fd = ff.factorize_remainder(desc, Ld["W1"], None, Ld["W2"], idx, seed=2024)
    torch.cuda.synchronize()
    got = {k: host(v) for k, v in fd.items() if v is not None}
    want = orc.factorize_remainder(L["W1"], L["W2"], None, idx_h, cfg.rank, seed=2024)
    for p, q in (("P1", "Q1"), ("P2", "Q2")):
        e = relf(got[p] @ got[q], want[p] @ want[q])
        assert e < 6e-3, (p, e)                      # two bf16-rounded factors
    split = ff.build_split(desc, Ld["W1"], None, Ld["W2"], idx, fd)
    X = wl.make_tokens(cfg, cfg.prefill_T)
    Y = guarded_forward(ff, desc, split, dev(X, "bf16"))
    torch.cuda.synchronize()
    ref = orc.forward_split(X, L["W1"], L["W2"], None, idx_h, "gelu", "lowrank", got)
    assert_close(host(Y), ref[0], "bf16", "C2 device factors, all rows")


def test_c2_opt13b_shape_65536_tokens(ff):
    """A batch sixteen times the benchmark's (more than 2^31 elements in h2's address range in
    bytes): index arithmetic at scale, checked on sampled rows against the oracle and on the
    first and last block of 4096 rows against a 4096-token call (rows are independent)."""
    cfg = C2
    L = wl.make_layer(cfg)
    Ld = layer_to_dev(L, cfg.dtype)
    idx_h = L["planted"]
    fac = wl.make_factors(cfg, L, idx_h)
    desc = desc_for(ff, cfg)
    split = ff.build_split(desc, Ld["W1"], None, Ld["W2"], torch.from_numpy(idx_h).cuda(),
                           {k: dev(v, "bf16") for k, v in fac.items()})
    T = 65536
    rows = sampled_rows(T, 16, seed=3)
    Xs = wl.make_tokens(cfg, 4096)
    Xd = dev(Xs, "bf16").repeat(T // 4096, 1)
    # make the sampled rows distinct from the repeats
    Xr = wl.make_tokens(cfg, len(rows), wl.gen.S_EVAL, layer=7)
    Xd[torch.from_numpy(rows).cuda()] = dev(Xr, "bf16")
    Y = ff.forward(desc, split, Xd)
    Y4 = guarded_forward(ff, desc, split, Xd[:4096].contiguous())
    torch.cuda.synchronize()
    ref = orc.forward_split(Xr, L["W1"], L["W2"], None, idx_h, "gelu", "lowrank", fac)[0]
    assert_close(host(Y[torch.from_numpy(rows).cuda()]), ref, "bf16", "C2 T=65536 sampled rows")
    keep = np.setdiff1d(np.arange(4096), rows)
    # (tile shapes and the split of the long reduction depend on T, so the sums are ordered
    # differently: equal up to the rounding of the bf16 intermediates, not bit for bit)
    assert relf(host(Y[:4096][torch.from_numpy(keep).cuda()]), host(Y4[torch.from_numpy(keep).cuda()])) < 3e-3
    blk = Y[4096 * 15:4096 * 16]
    keep15 = np.setdiff1d(keep, rows[rows >= 4096 * 15] - 4096 * 15)
    assert relf(host(blk[torch.from_numpy(keep15).cuda()]), host(Y4[torch.from_numpy(keep15).cuda()])) < 3e-3


def test_c3_llama7b_shape_prefill_and_decode(ff):
    cfg = C3
    L = wl.make_layer(cfg)
    Ld = layer_to_dev(L, cfg.dtype)
    Xc, scores, idx, idx_h = calibrate_and_select(ff, cfg, L, Ld, n_batches=2)
    # scores against the oracle on a sample of neurons (columns are independent), all 8192 tokens
    cols = np.concatenate([L["planted"][:16], np.random.default_rng(3).choice(cfg.d_ff, 48, replace=False)])
    acc_o = orc.score_accumulate(orc.new_accumulator(len(cols)), Xc, L["W1"][:, cols], L["Wg"][:, cols], "swiglu")
    assert_scores_close(scores.cpu().numpy()[cols], orc.neuron_scores(acc_o, L["W2"][cols, :]), "bf16",
                        "C3 sampled neurons")
    del Xc
    fac = wl.make_factors(cfg, L, idx_h)
    desc = desc_for(ff, cfg)
    split = ff.build_split(desc, Ld["W1"], Ld["Wg"], Ld["W2"], idx, {k: dev(v, "bf16") for k, v in fac.items()})
    del Ld
    torch.cuda.empty_cache()
    T = cfg.prefill_T
    X = wl.make_tokens(cfg, T)
    Y, Yh, Yr = guarded_forward(ff, desc, split, dev(X, "bf16"), want_parts=True)
    torch.cuda.synchronize()
    sw = {"W1h": L["W1"][:, idx_h].astype(np.float64), "Wgh": L["Wg"][:, idx_h].astype(np.float64),
          "W2h": L["W2"][idx_h, :].astype(np.float64)}

    def want_for(Xh):      # the two halves of Eq. 2 from the oracle (forward_split would also gather the unused dense rest)
        Y1 = orc.forward_heavy(Xh, sw, "swiglu")
        Y2 = orc.forward_remainder_lowrank(Xh, fac, "swiglu")
        return Y1 + Y2, Y1, Y2

    for g, w, nm in zip((Y, Yh, Yr), want_for(X), ("Y", "Y_heavy", "Y_rem")):               # all 4096 rows
        assert_close(host(g), w, "bf16", f"C3 T={T} {nm}")
    for B in cfg.decode_B:
        Xb = wl.make_tokens(cfg, B, wl.gen.S_EVAL, layer=B)
        Yb = guarded_forward(ff, desc, split, dev(Xb, "bf16"))
        torch.cuda.synchronize()
        assert_close(host(Yb), want_for(Xb)[0], "bf16", f"C3 decode B={B}")


def test_c4_llama7b_shape_int4_decode(ff):
    cfg = C4
    L = wl.make_layer(cfg)
    Ld = layer_to_dev(L, cfg.dtype)
    idx_h = L["planted"]                     # same recipe and heavy-set rule as the low-rank Llama-shaped layer
    desc = desc_for(ff, cfg)
    split = ff.build_split(desc, Ld["W1"], Ld["Wg"], Ld["W2"], torch.from_numpy(idx_h).cuda())
    sw = orc.split_weights(L["W1"], L["W2"], L["Wg"], idx_h)
    qw = orc.quantize_remainder(sw, cfg.group)
    for what, nm in ((0, "W1r"), (1, "Wgr"), (2, "W2r")):
        q, s = ff.split_export(desc, split, what)
        torch.cuda.synchronize()
        assert np.array_equal(q.cpu().numpy(), qw[nm][0]), nm
        assert np.array_equal(s.cpu().numpy().view(np.uint16), qw[nm][1].view(np.uint16)), nm
    for B in cfg.decode_B:
        Xb = wl.make_tokens(cfg, B, wl.gen.S_EVAL, layer=B)
        Yb, Yh, Yr = guarded_forward(ff, desc, split, dev(Xb, "bf16"), want_parts=True)
        torch.cuda.synchronize()
        Y1 = orc.forward_heavy(Xb, sw, "swiglu")
        Y2 = orc.forward_remainder_int4(Xb, qw, cfg.group, "swiglu")
        for g, w, nm in zip((Yb, Yh, Yr), (Y1 + Y2, Y1, Y2), ("Y", "Y_heavy", "Y_rem")):
            assert_close(host(g), w, "bf16", f"C4 int4 decode B={B} {nm}")


def test_c4_llama7b_shape_int4_many_tokens(ff):
    """4096 tokens through the int4 split (weights expanded to bf16, dense chain), all rows."""
    cfg = C4
    L = wl.make_layer(cfg)
    Ld = layer_to_dev(L, cfg.dtype)
    idx_h = L["planted"]
    desc = desc_for(ff, cfg)
    split = ff.build_split(desc, Ld["W1"], Ld["Wg"], Ld["W2"], torch.from_numpy(idx_h).cuda())
    del Ld
    T = 4096
    X = wl.make_tokens(cfg, T)
    Y, Yh, Yr = guarded_forward(ff, desc, split, dev(X, "bf16"), want_parts=True)
    torch.cuda.synchronize()
    sw = orc.split_weights(L["W1"], L["W2"], L["Wg"], idx_h)
    qw = orc.quantize_remainder(sw, cfg.group)
    Y1 = orc.forward_heavy(X, sw, "swiglu")
    Y2 = orc.forward_remainder_int4(X, qw, cfg.group, "swiglu")
    for g, w, nm in zip((Y, Yh, Yr), (Y1 + Y2, Y1, Y2), ("Y", "Y_heavy", "Y_rem")):
        assert_close(host(g), w, "bf16", f"C4 int4 T={T} {nm}")


def test_c4_llama7b_shape_w3h8(ff):
    """Sec. 5.2's pairing (heavy int8, remainder int3) at the Llama-2-7B shape: every code and
    scale, decode batches on the packed codes, and 4096 tokens on the expanded weights."""
    cfg = C4
    L = wl.make_layer(cfg)
    Ld = layer_to_dev(L, cfg.dtype)
    idx_h = L["planted"]
    desc = desc_for(ff, cfg, "w3h8")
    split = ff.build_split(desc, Ld["W1"], Ld["Wg"], Ld["W2"], torch.from_numpy(idx_h).cuda())
    del Ld
    sw = orc.split_weights(L["W1"], L["W2"], L["Wg"], idx_h)
    qr = orc.quantize_remainder(sw, 128, 3)
    qh = orc.quantize_heavy(sw, 128, 8)
    for what, src, nm in ((0, qr, "W1r"), (1, qr, "Wgr"), (2, qr, "W2r"), (3, qh, "W1h"), (4, qh, "Wgh"), (5, qh, "W2h")):
        q, s = ff.split_export(desc, split, what)
        torch.cuda.synchronize()
        assert np.array_equal(q.cpu().numpy(), src[nm][0]), nm
        assert np.array_equal(s.cpu().numpy().view(np.uint16), src[nm][1].view(np.uint16)), nm

    def want(X):
        Y1 = orc.forward_heavy_quant(X, qh, 128, "swiglu")
        Y2 = orc.forward_remainder_int4(X, qr, 128, "swiglu")
        return Y1 + Y2, Y1, Y2

    for B in (1, 16, 32):
        Xb = wl.make_tokens(cfg, B, wl.gen.S_EVAL, layer=B)
        got = guarded_forward(ff, desc, split, dev(Xb, "bf16"), want_parts=True)
        torch.cuda.synchronize()
        for g, w, nm in zip(got, want(Xb), ("Y", "Y_heavy", "Y_rem")):
            assert_close(host(g), w, "bf16", f"C4 w3h8 B={B} {nm}")
    T = 4096
    X = wl.make_tokens(cfg, T)
    Y = guarded_forward(ff, desc, split, dev(X, "bf16"))
    torch.cuda.synchronize()
    assert_close(host(Y), want(X)[0], "bf16", f"C4 w3h8 T={T}, all rows")


# ---------------------------------------------------------------- the 40-layer stack
# x <- x + FFN_l(n(x)), n = per-token RMS normalisation (the reading under which the stream of
# these synthetic layers stays finite).  Covered here, at full width (d_model 5120, d_ff 20480,
# k 819, rank 1280):
#   * ALL 40 layers teacher-forced: each layer is fed the oracle's own layer input.  Per layer:
#     the norm kernel, the scores of a 256-token calibration stream that the oracle moves
#     through the DENSE layers (heavy hitters are identified on the unmodified model), the
#     selected set, the split built from it, a 4096-token prefill whose first 64 rows are the
#     oracle's forward stream (moved through the SPLIT layers), a decode batch of 16, and one
#     step of the stack driver (norm + layer + residual, fp32 stream).
#   * layer 0: the full 16 384-token calibration (in four batches) against the oracle's scores
#     of every neuron.
#   * layers 0, 1, 20, 39: every one of the 4096 prefill rows against the oracle.
#   * the free-running 40-layer ffsplit_stack_forward call (T = 4096): its first 64 rows against
#     the oracle's end of stack (reported, and held to a looser bar: errors compound).
# The calibration stream past layer 0 has 256 tokens, not 16 384: the oracle's dense fp64 layers
# cost 0.42 GFLOP per token and layer.

C5_STATE = {}
C5_NC, C5_NF = 256, 64
C5_FULL_ROWS = (0, 1, 20, 39)


def _c5_layer(ff, layer, st):
    cfg = C5
    L = wl.make_layer(cfg, layer)
    Ld = layer_to_dev(L, cfg.dtype)
    desc0 = desc_for(ff, cfg, "none")
    # ---- the norm kernel on both oracle streams
    xn_cal_o = orc.token_rms_normalise(st["x_cal"])
    xn_fwd_o = orc.token_rms_normalise(st["x_fwd"])
    got_n = ff.token_rmsnorm(torch.from_numpy(st["x_cal"].astype(np.float32)).cuda(), ff.BF16)
    assert relf(host(got_n), xn_cal_o) < 3e-3, layer
    xn_cal = wl.bf16_round(xn_cal_o)            # the stored tokens both sides multiply
    xn_fwd = wl.bf16_round(xn_fwd_o)
    # ---- calibration on the dense layer: scores, selection
    scores, acc, tt = gpu_scores(ff, desc0, Ld, [dev(xn_cal[:100], "bf16"), dev(xn_cal[100:], "bf16")], reuse_tiled=True)
    idx, _, flag = ff.select_heavy(scores, cfg.k)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    assert int(flag.item()) == 0
    assert np.array_equal(idx_h, orc.select_heavy(scores.cpu().numpy(), cfg.k)), layer      # ranking kernel
    acc_o = orc.score_accumulate(orc.new_accumulator(cfg.d_ff), xn_cal, L["W1"], None, "gelu")
    want_s = orc.neuron_scores(acc_o, L["W2"])
    srt = np.sort(want_s)[::-1]
    margin = srt[cfg.k - 1] / srt[cfg.k]
    assert_scores_close(scores.cpu().numpy(), want_s, "bf16", f"C5 layer {layer}")
    # Past the first layer the stream is no longer isotropic (every token carries the mean
    # layer output), a few planted neurons go quiet and the heavy set is what the scores say:
    # the oracle's own selection, provided its cut is wider than the score error.
    # Where that cut is narrower than the score tolerance several sets are correct: compare what
    # is unique (every neuron clearly above the cut is selected, none clearly below it is) and
    # require exact equality wherever the cut is wide.
    cut, tol = srt[cfg.k - 1], 2 * 2e-2
    chosen = np.zeros(cfg.d_ff, bool)
    chosen[idx_h] = True
    assert chosen[want_s > cut * (1 + tol)].all(), layer
    assert not chosen[want_s < cut * (1 - tol)].any(), layer
    if margin > 1 + tol:
        assert np.array_equal(np.sort(idx_h), np.sort(orc.select_heavy(want_s, cfg.k))), layer
    else:
        diff = len(np.setxor1d(idx_h, orc.select_heavy(want_s, cfg.k)))
        st["narrow_cuts"].append((layer, round(float(margin), 5), diff))
    if layer == 0:
        assert np.array_equal(np.sort(idx_h), L["planted"])
        # the full calibration length: 16 384 tokens in four batches, every neuron's score
        Xc = wl.make_tokens(cfg, cfg.calib_T, wl.gen.S_CALIB)
        xs = [dev(Xc[i:i + 4096], "bf16") for i in range(0, cfg.calib_T, 4096)]
        s_full, _, tt = gpu_scores(ff, desc0, Ld, xs, reuse_tiled=True)
        assert tt == cfg.calib_T
        del xs
        acc_f = orc.new_accumulator(cfg.d_ff)
        for i in range(0, cfg.calib_T, 2048):
            orc.score_accumulate(acc_f, Xc[i:i + 2048], L["W1"], None, "gelu")
        want_f = orc.neuron_scores(acc_f, L["W2"])
        assert_scores_close(s_full.cpu().numpy(), want_f, "bf16", "C5 layer 0, 16384 tokens")
        i_full, _, _ = ff.select_heavy(s_full, cfg.k)
        assert np.array_equal(np.sort(i_full.cpu().numpy()), np.sort(orc.select_heavy(want_f, cfg.k)))
        assert np.array_equal(np.sort(i_full.cpu().numpy()), L["planted"])
        del Xc
    # ---- the split of this layer and its forward
    fac = wl.make_factors(cfg, L, idx_h, layer=layer)
    desc = desc_for(ff, cfg)
    split = ff.build_split(desc, Ld["W1"], None, Ld["W2"], idx, {k: dev(v, "bf16") for k, v in fac.items()})
    sw = {"W1h": L["W1"][:, idx_h].astype(np.float64), "W2h": L["W2"][idx_h, :].astype(np.float64), "Wgh": None}

    def want_for(Xh):
        return orc.forward_heavy(Xh, sw, "gelu") + orc.forward_remainder_lowrank(Xh, fac, "gelu")

    filler = wl.make_tokens(cfg, cfg.prefill_T - C5_NF, wl.gen.S_EVAL, layer=layer + 1)
    Xfull = np.concatenate([xn_fwd, filler])
    Y = guarded_forward(ff, desc, split, dev(Xfull, "bf16"))
    Yd = guarded_forward(ff, desc, split, dev(xn_fwd[:16], "bf16"))               # decode batch of 16
    torch.cuda.synchronize()
    want = want_for(xn_fwd)
    assert_close(host(Y[:C5_NF]), want, "bf16", f"C5 layer {layer} prefill, oracle stream rows")
    assert_close(host(Yd), want[:16], "bf16", f"C5 layer {layer} decode B=16")
    if layer in C5_FULL_ROWS:
        assert_close(host(Y), np.concatenate([want, want_for(filler)]), "bf16", f"C5 layer {layer} prefill, all rows")
    # one step of the stack driver on the oracle's stream: norm + layer + residual, fp32
    x_in = torch.from_numpy(st["x_fwd"].astype(np.float32)).cuda()
    x_out = ff.stack_forward(desc, [split], x_in.clone())
    torch.cuda.synchronize()
    assert_close(host(x_out), st["x_fwd"] + want, "bf16", f"C5 layer {layer} stack step")
    assert_close(host(x_out) - st["x_fwd"], want, "bf16", f"C5 layer {layer} stack step, update")
    st["splits"].append(split)
    # ---- both oracle streams move on (teacher forcing)
    st["x_fwd"] = st["x_fwd"] + want
    st["x_cal"] = st["x_cal"] + orc.dense_ffn(xn_cal, L["W1"], L["W2"], None, "gelu")
    st["done"] = layer + 1


@pytest.mark.parametrize("lo,hi", [(0, 8), (8, 16), (16, 24), (24, 32), (32, 40)],
                         ids=["layers0-7", "layers8-15", "layers16-23", "layers24-31", "layers32-39"])
def test_c5_opt13b_shape_stack_teacher_forced(ff, lo, hi):
    cfg = C5
    st = C5_STATE
    if not st:
        st.update({"x_cal": wl.make_tokens(cfg, C5_NC, wl.gen.S_CALIB).astype(np.float64),
                   "x_fwd": wl.make_tokens(cfg, C5_NF).astype(np.float64), "done": 0, "splits": [],
                   "narrow_cuts": [], "x0": None})
        st["x0"] = st["x_fwd"].copy()
    assert st["done"] == lo, "the layer groups of this test run in order (each starts where the last one stopped)"
    for layer in range(lo, hi):
        _c5_layer(ff, layer, st)
        print(f"[C5 stack] layer {layer} ok", flush=True)
    torch.cuda.empty_cache()


def test_c5_opt13b_shape_stack_free_running(ff):
    """The 40 splits built above in ONE ffsplit_stack_forward call at T = 4096: the first 64
    rows start from the oracle's stream and are compared with its end of stack."""
    cfg = C5
    st = C5_STATE
    assert st.get("done") == cfg.n_layers, "needs the 40 teacher-forced layers of the test above"
    desc = desc_for(ff, cfg)
    T = cfg.prefill_T
    x = np.concatenate([st["x0"], wl.make_tokens(cfg, T - C5_NF, wl.gen.S_EVAL, layer=77).astype(np.float64)])
    xd = torch.from_numpy(x.astype(np.float32)).cuda()
    g = Guarded(ff.workspace_bytes(desc, ff.WS_STACK, T))
    ff.stack_forward(desc, st["splits"], xd, workspace=g.view)
    g.check("stack_forward")
    got = host(xd[:C5_NF])
    e = relf(got, st["x_fwd"])
    print(f"[C5 stack] free-running end of stack, 40 layers: rel-Frobenius {e:.3e} vs the oracle's stream; "
          f"narrow cuts (layer, score ratio at the cut, size of the symmetric difference to the oracle's set): "
          f"{st['narrow_cuts']}", flush=True)
    assert torch.isfinite(xd).all()
    assert e < 3e-2            # per-layer errors of a few 1e-3 compound over 40 layers (not the graded bar)
    # a second call on the same input gives the same bits
    xd2 = torch.from_numpy(x.astype(np.float32)).cuda()
    ff.stack_forward(desc, st["splits"], xd2)
    torch.cuda.synchronize()
    assert torch.equal(xd, xd2)
    C5_STATE.clear()
    torch.cuda.empty_cache()


def test_c5_opt13b_shape_full_calibration_on_the_gpu(ff):
    """The whole calibration pass at its full size, on the device alone: 16 384 tokens through all 40
    dense layers (Sec. 4.2, first step), per layer the norm kernel, the score call in four batches
    of 4096 (the later ones reusing the re-tiled up projection), the selection, and the dense step
    through the stack driver.  The oracle cannot follow this in test time (about 275 TFLOP in fp64;
    the teacher-forced tests above compare every layer at 256 tokens and layer 0 at 16 384), so this
    checks what holds at any size: finite scores and stream, the planted set recovered (a few planted
    neurons go quiet past layer 0: at least 90 % of it), and a second run equal bit for bit.
    Layers are drawn on the device with the workload's recipe (seeded)."""
    cfg = C5
    T, nb = cfg.calib_T, 4
    desc = desc_for(ff, cfg, "dense")
    d, f, k = cfg.d_model, cfg.d_ff, cfg.k

    def layer(seed):
        g = torch.Generator(device="cuda").manual_seed(seed)
        planted = torch.sort(torch.randperm(f, generator=g, device="cuda")[:k]).values
        W1 = torch.randn((d, f), generator=g, device="cuda") * cfg.weight_std
        W2 = torch.randn((f, d), generator=g, device="cuda") * cfg.weight_std
        W1[:, planted] *= cfg.heavy_scale
        W2[planted, :] *= cfg.heavy_scale
        return W1.to(torch.bfloat16), W2.to(torch.bfloat16), planted

    def run():
        g = torch.Generator(device="cuda").manual_seed(99)
        x = torch.randn((T, d), generator=g, device="cuda")
        xn = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
        ws_s = torch.empty(ff.workspace_bytes(desc, ff.WS_SCORE, T // nb), dtype=torch.uint8, device="cuda")
        ws_f = torch.empty(ff.workspace_bytes(desc, ff.WS_STACK, T), dtype=torch.uint8, device="cuda")
        sets, recovered = [], []
        for l in range(cfg.n_layers):
            W1, W2, planted = layer(3000 + l)
            ff.token_rmsnorm(x, out=xn)
            acc = torch.zeros(2 * f, dtype=torch.float32, device="cuda")
            scores = torch.empty(f, dtype=torch.float32, device="cuda")
            tt = 0
            for b in range(nb):
                tt = ff.score_neurons(desc, xn[b * (T // nb):(b + 1) * (T // nb)], W1, None, W2, acc, tt,
                                      scores if b == nb - 1 else None, ff.SCORE_REUSE_TILED if b else 0, ws_s)
            idx, _, flag = ff.select_heavy(scores, k)
            split = ff.build_split(desc, W1, None, W2, idx)
            ff.stack_forward(desc, [split], x, workspace=ws_f)
            torch.cuda.synchronize()
            assert tt == T and int(flag.item()) == 0 and bool(torch.isfinite(scores).all())
            hit = int(torch.isin(idx.long(), planted).sum().item())
            recovered.append(hit / k)
            sets.append(idx.clone())
            del W1, W2, split
        assert bool(torch.isfinite(x).all())
        return x, sets, recovered

    x1, s1, rec = run()
    assert rec[0] == 1.0, rec[0]                      # isotropic input: exactly the planted set
    assert min(rec) >= 0.90, min(rec)
    x2, s2, _ = run()
    assert torch.equal(x1, x2) and all(torch.equal(a, b) for a, b in zip(s1, s2))
