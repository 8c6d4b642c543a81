"""GPU parity of the layer as the models wrap it: neuron biases, output bias and the residual
connection fused into ffsplit_forward_ex, the per-token RMS pre-norm, and the layer-stack
driver, each against the CPU oracle on the same seeded inputs."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import ffsplit_oracle as orc
import workloads as wl
from workloads.configs import C1, C2, C3, C4, C5, reduced
from gpu_util import TOL, dev, host, relf, assert_close, desc_for, layer_to_dev, Guarded

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ff():
    import paper_2401_04044_amd as m
    return m


def _biases(cfg, seed):
    rng = np.random.default_rng(seed)
    b1 = wl.gen.storage_round(rng.standard_normal(cfg.d_ff).astype(np.float32) * 0.5, cfg.dtype)
    b2 = rng.standard_normal(cfg.d_model).astype(np.float32) * 0.3
    return b1, b2


def _guarded_forward_ex(ff, desc, split, X, **kw):
    g = Guarded(ff.workspace_bytes(desc, ff.WS_FORWARD, X.shape[0]))
    out = ff.forward_ex(desc, split, X, workspace=g.view, **kw)
    g.check("forward_ex")
    return out


def f32_variant(cfg):
    return cfg.__class__(**{**cfg.__dict__, "dtype": "f32", "name": cfg.name + "-f32"})


EPI_CASES = [
    # name, cfg, remainder kind, tokens: every launch path of the chain (small batch one and two
    # token blocks, a few hundred rows with the reduction split, more than 1024 rows) and fp32
    ("lowrank_T5", reduced(C2, 320, 1111, rank=72), "lowrank", 5),
    ("lowrank_T40", reduced(C2, 320, 1111, rank=72), "lowrank", 40),
    ("lowrank_T200_split", reduced(C2, 1032, 1500, rank=520), "lowrank", 200),
    ("lowrank_T1300", reduced(C2, 256, 2100, rank=128), "lowrank", 1300),
    ("lowrank_T2100_wide", reduced(C5, 640, 2600, rank=192), "lowrank", 2100),
    ("dense_T7", reduced(C2, 256, 1000, rank=64), "dense", 7),
    ("dense_T300", reduced(C2, 256, 1000, rank=64), "dense", 300),
    ("dense_T1100", reduced(C2, 256, 1000, rank=64), "dense", 1100),
    ("none_T33", reduced(C2, 256, 1000, rank=64), "none", 33),
    ("none_T1500", reduced(C2, 256, 1000, rank=64), "none", 1500),
    ("f32_lowrank_T77", f32_variant(reduced(C1, 96, 300, rank=24)), "lowrank", 77),
    ("f32_dense_T130", f32_variant(reduced(C1, 96, 300, rank=24)), "dense", 130),
]


@pytest.mark.parametrize("name,cfg,kind,T", EPI_CASES, ids=[c[0] for c in EPI_CASES])
def test_forward_ex_biases_and_residual_match_oracle(ff, name, cfg, kind, T):
    L = wl.make_layer(cfg)
    idx = L["planted"][::-1].copy()
    fac = wl.make_factors(cfg, L, idx) if kind == "lowrank" else None
    b1, b2 = _biases(cfg, 11)
    X = wl.make_tokens(cfg, T)
    res = np.random.default_rng(12).standard_normal((T, cfg.d_model)).astype(np.float32) * 3.0
    Ld = layer_to_dev(L, cfg.dtype)
    desc = desc_for(ff, cfg, kind)
    idx_d = torch.from_numpy(idx).cuda()
    fd = None if fac is None else {k: dev(v, cfg.dtype) for k, v in fac.items()}
    split = ff.build_split(desc, Ld["W1"], None, Ld["W2"], idx_d, fd)
    b1p = ff.pack_neuron_bias(desc, dev(b1, cfg.dtype), idx_d)
    b2d = torch.from_numpy(b2).cuda()
    resd = torch.from_numpy(res).cuda()
    Xd = dev(X, cfg.dtype)
    want, w1, w2 = orc.forward_split_biased(X, L["W1"], L["W2"], idx, kind, fac, b1, b2, res)
    # everything at once, fp32 destination, the two halves on the side
    Y, Yh, Yr = _guarded_forward_ex(ff, desc, split, Xd, b1_packed=b1p, b2=b2d, residual=resd, y_f32=True,
                                    want_parts=True)
    torch.cuda.synchronize()
    assert Y.dtype == torch.float32
    assert_close(host(Y), want, cfg.dtype, f"{name} Y")
    assert_close(host(Y) - res, want - res, cfg.dtype, f"{name} Y - residual")     # the layer's own part
    assert_close(host(Yh), w1, cfg.dtype, f"{name} Y_heavy")
    if np.linalg.norm(w2) > 0:
        assert_close(host(Yr), w2, cfg.dtype, f"{name} Y_rem")
    # in place on the stream: Y is the residual buffer
    stream = resd.clone()
    _guarded_forward_ex(ff, desc, split, Xd, Y=stream, b1_packed=b1p, b2=b2d, residual=stream, y_f32=True)
    torch.cuda.synchronize()
    assert torch.equal(stream, Y)
    # storage-type destination; and each addition on its own
    Yb = _guarded_forward_ex(ff, desc, split, Xd, b1_packed=b1p, b2=b2d, residual=resd)
    assert Yb.dtype == Xd.dtype
    assert_close(host(Yb), want, cfg.dtype, f"{name} Y in the storage type")
    only_b1 = _guarded_forward_ex(ff, desc, split, Xd, b1_packed=b1p)
    assert_close(host(only_b1), orc.forward_split_biased(X, L["W1"], L["W2"], idx, kind, fac, b1)[0], cfg.dtype,
                 f"{name} b1 only")
    only_b2 = _guarded_forward_ex(ff, desc, split, Xd, b2=b2d)
    assert_close(host(only_b2), orc.forward_split_biased(X, L["W1"], L["W2"], idx, kind, fac, None, b2)[0], cfg.dtype,
                 f"{name} b2 only")
    # no additions: the plain entry point, bit for bit
    plain = ff.forward(desc, split, Xd)
    none = _guarded_forward_ex(ff, desc, split, Xd)
    torch.cuda.synchronize()
    assert torch.equal(plain, none)


def test_neuron_bias_is_packed_in_the_split_order(ff):
    cfg = reduced(C2, 128, 333, rank=32)
    L = wl.make_layer(cfg)
    idx = L["planted"][::-1].copy()
    b1, _ = _biases(cfg, 3)
    desc = desc_for(ff, cfg, "lowrank")
    got = ff.pack_neuron_bias(desc, dev(b1, "bf16"), torch.from_numpy(idx).cuda()).cpu().numpy()
    k, m = len(idx), cfg.d_ff - len(idx)
    kp, mp = -(-k // 64) * 64, -(-m // 64) * 64
    assert got.shape == (kp + mp,)
    perm = orc.neuron_permutation(idx, cfg.d_ff)
    assert np.array_equal(got[:k], b1[perm[:k]]) and not got[k:kp].any()
    assert np.array_equal(got[kp:kp + m], b1[perm[k:]]) and not got[kp + m:].any()


GATED_CASES = [
    ("swiglu_lowrank_T9", reduced(C3, 192, 700, rank=64), "lowrank", 9),
    ("swiglu_lowrank_T1059", reduced(C3, 192, 1500, rank=64), "lowrank", 1059),
    ("int4_T4", reduced(C4, 256, 700), "int4", 4),
    ("int4_T21", reduced(C4, 384, 1000), "int4", 21),
    ("int4_T300", reduced(C4, 256, 700), "int4", 300),
    ("w3h8_T7", reduced(C4, 256, 700), "w3h8", 7),
    ("w3h8_T40", reduced(C4, 256, 700), "w3h8", 40),
    ("w3h8_T200", reduced(C4, 384, 1000), "w3h8", 200),
]


@pytest.mark.parametrize("name,cfg,kind,T", GATED_CASES, ids=[c[0] for c in GATED_CASES])
def test_forward_ex_output_bias_and_residual_on_gated_and_quantised_layers(ff, name, cfg, kind, T):
    """No neuron biases there (the gated layers carry none): b2, the residual and the fp32
    destination ride on the last product of every remainder kind."""
    L = wl.make_layer(cfg)
    idx = L["planted"]
    fac = wl.make_factors(cfg, L, idx) if kind == "lowrank" else None
    _, b2 = _biases(cfg, 21)
    X = wl.make_tokens(cfg, T)
    res = np.random.default_rng(22).standard_normal((T, cfg.d_model)).astype(np.float32) * 2.0
    Ld = layer_to_dev(L, "bf16")
    desc = desc_for(ff, cfg, kind)
    fd = None if fac is None else {k: dev(v, "bf16") for k, v in fac.items()}
    split = ff.build_split(desc, Ld["W1"], Ld["Wg"], Ld["W2"], torch.from_numpy(idx).cuda(), fd)
    want = orc.forward_split(X, L["W1"], L["W2"], L["Wg"], idx, cfg.act, kind, fac, group=128)[0]
    want = res + want + b2[None, :]
    b2d, resd = torch.from_numpy(b2).cuda(), torch.from_numpy(res).cuda()
    Y = _guarded_forward_ex(ff, desc, split, dev(X, "bf16"), b2=b2d, residual=resd, y_f32=True)
    torch.cuda.synchronize()
    assert_close(host(Y), want, "bf16", f"{name} Y")
    assert_close(host(Y) - res, want - res, "bf16", f"{name} Y - residual")
    Yb = _guarded_forward_ex(ff, desc, split, dev(X, "bf16"), b2=b2d, residual=resd)
    assert_close(host(Yb), want, "bf16", f"{name} Y in bf16")
    # neuron biases are refused there
    b1p = torch.zeros(int(ff.lib.ffsplit_neuron_bias_floats(ctypes.byref(desc))), dtype=torch.float32, device="cuda")
    with pytest.raises(ff.FFSplitError) as e:
        ff.forward_ex(desc, split, dev(X, "bf16"), b1_packed=b1p)
    assert e.value.code == -6


@pytest.mark.parametrize("T,d", [(1, 64), (37, 328), (300, 5120), (5, 8), (3, 10240)])
def test_token_rmsnorm_matches_oracle(ff, T, d):
    x = (np.random.default_rng(T).standard_normal((T, d)) * np.linspace(0.01, 40.0, T)[:, None]).astype(np.float32)
    if T > 2:
        x[2] = 0.0                                         # an all-zero token stays zero (eps)
    want = orc.token_rms_normalise(x)
    xd = torch.from_numpy(x).cuda()
    got32 = ff.token_rmsnorm(xd, ff.F32).cpu().numpy().astype(np.float64)
    got16 = ff.token_rmsnorm(xd, ff.BF16).float().cpu().numpy().astype(np.float64)
    assert np.abs(got32 - want).max() <= 2e-6 * np.abs(want).max()
    # bf16: one rounding of the fp32 result
    assert np.array_equal(got16, wl.bf16_round(got32.astype(np.float32)).astype(np.float64))
    assert relf(got16, want) < 3e-3


def _stack_layers(ff, cfg, n_layers, with_bias):
    """Per layer: weights, planted heavy set, factors, biases; packed on the device."""
    layers = []
    for l in range(n_layers):
        L = wl.make_layer(cfg, l)
        idx = L["planted"]
        fac = wl.make_factors(cfg, L, idx, layer=l)
        b1, b2 = _biases(cfg, 100 + l) if with_bias else (None, None)
        Ld = layer_to_dev(L, cfg.dtype)
        desc = desc_for(ff, cfg, "lowrank")
        idx_d = torch.from_numpy(idx).cuda()
        split = ff.build_split(desc, Ld["W1"], None, Ld["W2"], idx_d, {k: dev(v, cfg.dtype) for k, v in fac.items()})
        b1p = ff.pack_neuron_bias(desc, dev(b1, cfg.dtype), idx_d) if with_bias else None
        b2d = torch.from_numpy(b2).cuda() if with_bias else None
        layers.append({"L": L, "idx": idx, "fac": fac, "b1": b1, "b2": b2, "split": split, "b1p": b1p, "b2d": b2d})
    return layers


@pytest.mark.parametrize("with_bias,T", [(False, 100), (True, 100), (False, 1300), (True, 20)])
def test_stack_forward_matches_oracle(ff, with_bias, T):
    """x <- x + FFN_split(n(x)) over 6 layers of a scaled-down 40-layer-stack shape: every layer
    teacher-forced on the oracle's stream, and the free-running end of the stack."""
    cfg = reduced(C5, 256, 1000, rank=64)
    n_layers = 6
    layers = _stack_layers(ff, cfg, n_layers, with_bias)
    desc = desc_for(ff, cfg, "lowrank")
    x0 = wl.make_tokens(cfg, T).astype(np.float64) * 2.0
    # oracle stream (its layer inputs are what teacher forcing feeds)
    xs = [x0]
    for ly in layers:
        xn = wl.bf16_round(orc.token_rms_normalise(xs[-1]))       # the stored, rounded tokens both sides multiply
        Yl = orc.forward_split_biased(xn, ly["L"]["W1"], ly["L"]["W2"], ly["idx"], "lowrank", ly["fac"], ly["b1"],
                                      ly["b2"], xs[-1])[0]
        xs.append(Yl)
    for l, ly in enumerate(layers):
        xin = torch.from_numpy(xs[l].astype(np.float32)).cuda()
        out = ff.stack_forward(desc, [ly["split"]], xin.clone(), [ly["b1p"]] if with_bias else None,
                               [ly["b2d"]] if with_bias else None)
        torch.cuda.synchronize()
        assert_close(host(out), xs[l + 1], "bf16", f"stack layer {l} teacher-forced")
        assert_close(host(out) - xs[l], xs[l + 1] - xs[l], "bf16", f"stack layer {l} update")
    g = Guarded(ff.workspace_bytes(desc, ff.WS_STACK, T))
    x = torch.from_numpy(x0.astype(np.float32)).cuda()
    ff.stack_forward(desc, [ly["split"] for ly in layers], x, [ly["b1p"] for ly in layers] if with_bias else None,
                     [ly["b2d"] for ly in layers] if with_bias else None, workspace=g.view)
    g.check("stack_forward")
    assert_close(host(x), xs[-1], "bf16", "stack free-running end")


GRAPH_CASES = [
    # name, cfg, remainder kind, tokens: prefill chain, small-batch chain, int4 decode, W3H8 decode
    ("lowrank_T1300", reduced(C5, 256, 1000, rank=64), "lowrank", 1300),
    ("lowrank_T16", reduced(C5, 256, 1000, rank=64), "lowrank", 16),
    ("int4_T16", reduced(C4, 256, 768), "int4", 16),
    ("w3h8_T16", reduced(C4, 256, 768), "w3h8", 16),
]


@pytest.mark.parametrize("name,cfg,kind,T", GRAPH_CASES, ids=[c[0] for c in GRAPH_CASES])
def test_stack_and_forward_replay_from_a_hip_graph(ff, name, cfg, kind, T):
    """The calls launch kernels only (no allocation, no synchronisation, no memset): a caller may
    capture them.  Three layers of the stack driver resp. one forward are captured once and replayed
    three times, with eager work and synchronisations of the program's own between the replays;
    every replay must equal the eager result bit for bit."""
    gated = cfg.act == "swiglu"
    L = wl.make_layer(cfg, 0)
    idx = L["planted"]
    Ld = layer_to_dev(L, cfg.dtype)
    desc = desc_for(ff, cfg, kind)
    fac = wl.make_factors(cfg, L, idx) if kind == "lowrank" else None
    split = ff.build_split(desc, Ld["W1"], Ld["Wg"] if gated else None, Ld["W2"], torch.from_numpy(idx).cuda(),
                           {k: dev(v, cfg.dtype) for k, v in fac.items()} if fac else None)
    x0 = torch.from_numpy((wl.make_tokens(cfg, T) * 2.0).astype(np.float32)).cuda()
    use_stack = kind == "lowrank"
    if use_stack:
        ws = torch.empty(ff.workspace_bytes(desc, ff.WS_STACK, T), dtype=torch.uint8, device="cuda")
        x = x0.clone()

        def step():
            ff.stack_forward(desc, [split, split, split], x, workspace=ws)
    else:
        ws = torch.empty(ff.workspace_bytes(desc, ff.WS_FORWARD, T), dtype=torch.uint8, device="cuda")
        xb = x0.to(torch.bfloat16)
        x = torch.empty((T, cfg.d_model), dtype=torch.bfloat16, device="cuda")

        def step():
            ff.forward(desc, split, xb, x, False, ws)
    # eager result (also the warm-up that sets the kernels' one-time attributes before the capture)
    step()
    torch.cuda.synchronize()
    want = x.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        if use_stack:
            x.copy_(x0)
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        if use_stack:
            x.copy_(x0)            # eager work between the replays
        else:
            x.zero_()
        ws.random_(0, 255)         # the workspace holds nothing a later call relies on
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(x, want), f"replay {rep} differs from the eager result"


def test_stack_calibration_runs_on_the_gpu():
    """The calibration pass of a layer stack on the device alone (Sec. 4.2, first step: heavy hitters
    are found on the unmodified model): per layer the library's norm kernel, the score call on the
    normalised tokens, the selection, and the step x <- x + FFN_dense(n(x)) through the stack driver
    on the exact dense layer (k heavy neurons + dense remainder).  Free-running over six layers of a
    scaled-down 40-layer-stack shape; scores, heavy sets and the propagated stream against the
    oracle's calibration chain."""
    from gpu_util import assert_scores_close
    cfg = reduced(C5, 256, 1000, rank=64)
    n_layers, T = 6, 600
    ffm = ff_mod()
    desc = desc_for(ffm, cfg, "dense")
    x_o = wl.make_tokens(cfg, T, wl.gen.S_CALIB).astype(np.float64) * 2.0
    x_d = torch.from_numpy(x_o.astype(np.float32)).cuda()
    xn_d = torch.empty((T, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    for l in range(n_layers):
        L = wl.make_layer(cfg, l)
        Ld = layer_to_dev(L, cfg.dtype)
        # oracle: scores on the normalised tokens (rounded as stored), then the dense step
        xn_o = wl.bf16_round(orc.token_rms_normalise(x_o))
        acc_o = orc.score_accumulate(orc.new_accumulator(cfg.d_ff), xn_o, L["W1"], None, "gelu")
        want_scores = orc.neuron_scores(acc_o, L["W2"])
        want_idx = orc.select_heavy(want_scores, cfg.k)
        x_o = x_o + orc.dense_ffn(xn_o, L["W1"], L["W2"], None, "gelu")
        # device
        ffm.token_rmsnorm(x_d, out=xn_d)
        acc = torch.zeros(2 * cfg.d_ff, dtype=torch.float32, device="cuda")
        scores = torch.empty(cfg.d_ff, dtype=torch.float32, device="cuda")
        ffm.score_neurons(desc, xn_d, Ld["W1"], None, Ld["W2"], acc, 0, scores)
        idx, _, flag = ffm.select_heavy(scores, cfg.k)
        split = ffm.build_split(desc, Ld["W1"], None, Ld["W2"], idx)
        ffm.stack_forward(desc, [split], x_d)
        torch.cuda.synchronize()
        assert int(flag.item()) == 0
        assert_scores_close(host(scores), want_scores, "bf16", f"stack calibration layer {l}")
        assert np.array_equal(np.sort(idx.cpu().numpy()), np.sort(want_idx)), f"heavy set of layer {l}"
        assert_close(host(x_d), x_o, "bf16", f"stack calibration stream after layer {l}")


def ff_mod():
    import paper_2401_04044_amd as m
    return m
