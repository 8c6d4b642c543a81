"""The input generators: determinism, storage rounding, the planted set and the
factor inputs (Eckart-Young closed form for the truncated factors)."""
import numpy as np

import workloads as wl
from workloads.configs import C1, C2, C3, C4, C5, reduced


def test_configs_follow_k_rule_and_work_counts():
    for c in (C1, C2, C3, C4, C5):
        assert c.k == int(round(c.heavy_frac * c.d_ff))
        assert len(wl.planted_set(c)) == c.k
    assert abs(C2.flops_per_token() - 22.48e6) < 0.01e6
    assert abs(C3.flops_per_token() - 102.9e6) < 0.1e6
    assert abs(C5.flops_per_token() - 143.7e6) < 0.1e6
    assert abs(C4.weight_bytes() - 79.78e6) < 0.02e6
    assert abs(C3.weight_bytes() - 102.9e6) < 0.1e6


def test_bf16_round_is_rne_and_idempotent():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -9, -1.0 - 2 ** -8, 3.1415926, 0.0, -0.0],
                 np.float32)
    r = wl.bf16_round(x)
    assert r[0] == 1.0 and r[1] == 1.0                     # tie -> even (1.0)
    assert r[2] == np.float32(1.0 + 4 * 2 ** -8)           # tie -> even (up)
    assert r[3] == 1.0 and r[4] == -1.0
    assert np.array_equal(wl.bf16_round(r), r)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    import torch
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(t, r)


def test_layer_is_seeded_and_planted_columns_scaled():
    cfg = reduced(C3, 64, 256, rank=16)
    a, b = wl.make_layer(cfg), wl.make_layer(cfg)
    for nm in ("W1", "W2", "Wg"):
        assert np.array_equal(a[nm], b[nm])
        assert np.array_equal(wl.bf16_round(a[nm]), a[nm])
    p = a["planted"]
    rest = wl.remainder_order(p, cfg.d_ff)
    assert len(p) == cfg.k and len(rest) == cfg.m and not set(p) & set(rest)
    assert a["W1"][:, p].std() / a["W1"][:, rest].std() > 5
    assert a["W2"][p, :].std() / a["W2"][rest, :].std() > 5
    assert not np.array_equal(wl.make_layer(cfg, layer=1)["W1"], a["W1"])
    x = wl.make_tokens(cfg, 7)
    assert x.shape == (7, 64) and np.array_equal(wl.make_tokens(cfg, 7), x)


def test_truncated_factors_eckart_young():
    rng = np.random.default_rng(0)
    for shape in ((12, 40), (40, 12)):
        W = rng.standard_normal(shape)
        sv = np.linalg.svd(W, compute_uv=False)
        for r in (1, 5, 12):
            P, Q = wl.truncated_factors(W, r)
            assert P.shape == (shape[0], r) and Q.shape == (r, shape[1])
            err = np.linalg.norm(W - P @ Q) ** 2
            assert np.isclose(err, np.sum(sv[r:] ** 2), rtol=1e-9, atol=1e-10)
            # balanced: both factors carry sqrt(sigma)
            assert np.allclose(np.linalg.norm(P, axis=0) ** 2, sv[:r], rtol=1e-8)
            assert np.allclose(np.linalg.norm(Q, axis=1) ** 2, sv[:r], rtol=1e-8)


def test_make_factors_shapes_and_rounding():
    cfg = reduced(C3, 32, 96, rank=8)
    L = wl.make_layer(cfg)
    f = wl.make_factors(cfg, L, L["planted"])
    m = cfg.m
    assert f["P1"].shape == (32, 8) and f["Q1"].shape == (8, m)
    assert f["Pg"].shape == (32, 8) and f["Qg"].shape == (8, m)
    assert f["P2"].shape == (m, 8) and f["Q2"].shape == (8, 32)
    assert np.array_equal(wl.bf16_round(f["Q1"]), f["Q1"])
    g = wl.make_factors(reduced(C5, 32, 96, rank=8), wl.make_layer(reduced(C5, 32, 96, rank=8)),
                        L["planted"][:4])
    assert g["Pg"] is None and g["P1"].shape == (32, 8)
