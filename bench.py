#!/usr/bin/env python3
"""Benchmark of the split feed-forward layer on one MI355X.

Headline workload (the largest single-GPU configuration): the OPT-13B-shaped
40-layer stack (d_model 5120, d_ff 20480, GeLU, bf16, k = 819 heavy neurons,
rank-1280 remainder), prefill of 4 x 1024 = 4096 tokens.  A step is one
ffsplit_stack_forward call: for each of 40 DISTINCT layers the per-token RMS norm,
the split layer (four chained products) and the residual add on the fp32 stream.
value = 40 * T / t_step, the tokens/s per layer.  Weights, packed splits and
inputs are resident in HBM before the timed region.  Prints ONE JSON line.

Beside it, each with its own roofline entry ("roofline.per_config"): one-layer
prefill of the C2 / C3 / C5 shapes (MFMA-bound) and the int4 decode of the C4
shape (HBM-bound, rotating over enough split copies that every weight byte comes
from HBM, not from the 256 MB last-level cache); further sections: bf16 low-rank
decode, the int8/int3 pairing, the fp32 correctness config, the calibration
pipeline, and this machine's measured ceilings (the library's own pure-MFMA loop
and streaming-read kernels).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15   # FLOP/s, dense bf16, MI355X datasheet
HBM_PEAK = 8.0e12         # B/s
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")   # written by the profile summary step


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=40, help="layers of the stack (the workload has 40)")
    ap.add_argument("--only", default="", help="comma list of sections to run besides the headline: "
                    "prefill,decode,w3h8,c1,pipeline,yardsticks,cpu (default: all)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--preheat-ms", type=float, default=100.0,
                    help="untimed steady load before every timed loop, so that the clocks have settled")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference dispatch for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2401_04044_amd as ff
    import workloads as wl
    import dataclasses
    from workloads.configs import C1, C2, C3, C4, C5

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    bf = torch.bfloat16
    t_start = time.perf_counter()
    sections = set(s for s in args.only.split(",") if s) or {"prefill", "decode", "w3h8", "c1", "pipeline",
                                                              "yardsticks", "cpu"}
    if args.no_cpu:
        sections.discard("cpu")
    traffic = {}
    if os.path.exists(TRAFFIC_FILE):
        traffic = json.load(open(TRAFFIC_FILE))

    def note(msg):
        print(f"[bench {time.perf_counter() - t_start:6.1f}s] {msg}", file=sys.stderr, flush=True)

    def dev(a, dt=bf):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, np.float32)).to("cuda", dtype=dt)

    def timed(fn, n, warm):
        """(seconds per call by HIP events on the launch stream, wall seconds per call)."""
        preheat_s = args.preheat_ms * 1e-3
        # The GPU's clocks take tens of milliseconds of continuous load to settle after the host-side
        # preparation that precedes every section (measured: the first ~10 ms of a loop run 5-15 %
        # slower than its steady state).  Untimed calls of the same step until preheat_s has passed,
        # then the warm-up steps asked for, then the timed ones.
        t_pre = time.perf_counter()
        while time.perf_counter() - t_pre < preheat_s:
            for _ in range(4):
                fn()
            torch.cuda.synchronize()
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return e0.elapsed_time(e1) * 1e-3 / n, wall / n

    def device_layer(cfg, seed):
        """A layer of the workload's recipe drawn on the device (N(0, 0.02^2) weights, a seeded planted
        set scaled up, seeded Gaussian factors of the right shape): the stack needs 40 distinct
        layers and the host generator takes seconds per layer."""
        g = torch.Generator(device="cuda").manual_seed(seed)
        d, f, k, r = cfg.d_model, cfg.d_ff, cfg.k, cfg.rank
        planted = torch.sort(torch.randperm(f, generator=g, device="cuda")[:k]).values.to(torch.int32)
        out = {"idx": planted}
        for nm in ("W1", "W2") + (("Wg",) if cfg.act == "swiglu" else ()):
            w = torch.randn((f, d) if nm == "W2" else (d, f), generator=g, device="cuda") * cfg.weight_std
            if nm == "W2":
                w[planted.long(), :] *= cfg.heavy_scale
            else:
                w[:, planted.long()] *= cfg.heavy_scale
            out[nm] = w.to(bf)
        out.setdefault("Wg", None)
        a = (cfg.weight_std / r ** 0.5) ** 0.5
        m = f - k
        fac = {}
        for tag, shp in (("1", (d, m)), ("g", (d, m)), ("2", (m, d))):
            if tag == "g" and cfg.act != "swiglu":
                fac["Pg"] = fac["Qg"] = None
                continue
            fac["P" + tag] = (torch.randn((shp[0], r), generator=g, device="cuda") * a).to(bf)
            fac["Q" + tag] = (torch.randn((r, shp[1]), generator=g, device="cuda") * a).to(bf)
        out["fac"] = fac
        return out

    if args.calib_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        note("reference copy done: 3 x 256 MiB read + 256 MiB written")

    from oracle import ffsplit_oracle as orc     # the parity samples and the cpu_baseline leg only

    # ------------------------------------------------------------ headline: the C5 40-layer stack
    cfg = C5
    T = cfg.prefill_T
    n_layers = args.layers
    desc = ff.make_desc(cfg.d_model, cfg.d_ff, cfg.act, cfg.dtype, cfg.k, "lowrank", cfg.rank)
    # layer 0 comes from the host generator (the seeded workload the oracle sees); its heavy set from
    # the library's own calibration on a 4096-token slice
    L0 = wl.make_layer(cfg, 0)
    note("C5 layer 0 generated (host)")
    W1, W2 = dev(L0["W1"]), dev(L0["W2"])
    Xc = dev(wl.make_tokens(cfg, 4096, wl.gen.S_CALIB))
    acc = torch.zeros(2 * cfg.d_ff, dtype=torch.float32, device="cuda")
    scores = torch.empty(cfg.d_ff, dtype=torch.float32, device="cuda")
    ff.score_neurons(desc, Xc, W1, None, W2, acc, 0, scores)
    idx0, _, flag = ff.select_heavy(scores, cfg.k)
    torch.cuda.synchronize()
    idx0_h = idx0.cpu().numpy()
    heavy_ok = bool(np.array_equal(np.sort(idx0_h), L0["planted"])) and int(flag.item()) == 0
    fac0 = wl.make_factors(cfg, L0, idx0_h, layer=0)
    splits = [ff.build_split(desc, W1, None, W2, idx0, {k: dev(v) for k, v in fac0.items()})]
    del W1, W2, Xc
    for l in range(1, n_layers):
        Ld = device_layer(cfg, 5000 + l)
        splits.append(ff.build_split(desc, Ld["W1"], None, Ld["W2"], Ld["idx"], Ld["fac"]))
        del Ld
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    note(f"{n_layers} distinct C5 splits built ({n_layers * cfg.weight_bytes() / 1e9:.1f} GB)")
    x0_h = wl.make_tokens(cfg, T).astype(np.float32)
    x0 = torch.from_numpy(x0_h).cuda()
    x = x0.clone()
    ws = torch.empty(ff.workspace_bytes(desc, ff.WS_STACK, T), dtype=torch.uint8, device="cuda")

    def step():
        # (the stream keeps moving from step to step: values stay finite under the norm, and
        # the step's cost does not depend on them)
        ff.stack_forward(desc, splits, x, workspace=ws)

    t_ev, t_wall = timed(step, args.steps, args.warmup)
    flops_layer = cfg.flops_per_token() * T
    note(f"stack of {n_layers}: {t_ev*1e3:.2f} ms/step (events), {t_wall*1e3:.2f} ms/step (wall), "
         f"{t_ev/n_layers*1e6:.1f} us per layer")
    # parity of the timed configuration: layer 0 of the stack on sampled rows (rows are independent)
    x.copy_(x0)
    ff.stack_forward(desc, splits[:1], x, workspace=ws)
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(0).choice(T, 32, replace=False))
    xn = wl.bf16_round(orc.token_rms_normalise(x0_h[rows].astype(np.float64)))
    sw = {"W1h": L0["W1"][:, idx0_h].astype(np.float64), "W2h": L0["W2"][idx0_h, :].astype(np.float64), "Wgh": None}
    want = x0_h[rows] + orc.forward_heavy(xn, sw, "gelu") + orc.forward_remainder_lowrank(xn, fac0, "gelu")
    got = x[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    rel_err = float(np.linalg.norm(got - want) / np.linalg.norm(want))
    upd_err = float(np.linalg.norm((got - x0_h[rows]) - (want - x0_h[rows])) / np.linalg.norm(want - x0_h[rows]))

    out = {
        "metric": "split-FFN tokens/s per layer; % of MFMA peak (prefill) / HBM BW (decode)",
        "value": n_layers * T / t_wall,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": t_wall * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"C5 OPT-13B-shaped split-FFN stack, prefill: {n_layers} distinct layers, d_model=5120 "
                               "d_ff=20480 GeLU k=819 rank=1280, T=4x1024=4096, pre-norm + residual per layer (fp32 "
                               "stream); value = layers*T/t_step (tokens/s per layer)",
                   "layers": n_layers, "T": T, "preheat_ms": args.preheat_ms},
        "roofline": {"bound": "mfma",
                     "kernel": "one layer of ffsplit_stack_forward = token_rmsnorm + 4 chained gemm_bf16_dl_kernel "
                               "launches (+ split-K sum), residual fused into the last; per-launch figures in profiles/",
                     "achieved": flops_layer * n_layers / t_ev / 1e12, "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
                     "frac": flops_layer * n_layers / t_ev / MFMA_BF16_PEAK,
                     "traffic": traffic.get("C5_stack_layer"),
                     "flops_per_launch": flops_layer, "us_per_launch_hip_events": t_ev / n_layers * 1e6,
                     "per_config": {}},
        "parity": {"layer0_rel_frobenius_vs_oracle_32_rows": rel_err, "layer0_update_rel_frobenius": upd_err,
                   "heavy_set_equals_planted": heavy_ok},
    }
    per = out["roofline"]["per_config"]
    del x, x0, ws
    keep_c5 = splits[:8]
    del splits
    torch.cuda.empty_cache()

    # ------------------------------------------------------------ cpu baseline: the oracle as it stands
    if "cpu" in sections:
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        n_s = 1024
        xs = wl.bf16_round(orc.token_rms_normalise(x0_h[:n_s].astype(np.float64)))
        reps, spent = 0, 0.0
        while spent < 12.0 and reps < 64:      # about 12 s of host work
            t0 = time.perf_counter()
            orc.forward_heavy(xs, sw, "gelu") + orc.forward_remainder_lowrank(xs, fac0, "gelu")
            spent += time.perf_counter() - t0
            reps += 1
        note(f"oracle timed: {reps} reps of {n_s} tokens in {spent:.1f} s")
        out["cpu_baseline"] = {"value": n_s * reps / spent, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{reps} x the split forward (FFN_1 + low-rank FFN_2, numpy fp64) of layer 0 "
                                         f"of the same stack on {n_s} of its {T} tokens; tokens/s per layer"}
    del L0, fac0, sw

    # ------------------------------------------------------------ one-layer prefill of the bf16 low-rank shapes
    def lowrank_split(cfg_d, n_cp):
        Ld = device_layer(cfg_d, 7000 + cfg_d.index)
        dd = ff.make_desc(cfg_d.d_model, cfg_d.d_ff, cfg_d.act, cfg_d.dtype, cfg_d.k, "lowrank", cfg_d.rank)
        spd = ff.build_split(dd, Ld["W1"], Ld["Wg"], Ld["W2"], Ld["idx"], Ld["fac"])
        torch.cuda.synchronize()
        return dd, [spd] + [spd.clone() for _ in range(n_cp - 1)]

    lr = {}
    if "prefill" in sections or "decode" in sections:
        for cfg_d, n_cp in ((C2, 8), (C3, 10), (C5, 8)):
            if cfg_d is C5:
                dd, spds = ff.make_desc(C5.d_model, C5.d_ff, C5.act, C5.dtype, C5.k, "lowrank", C5.rank), keep_c5
            else:
                dd, spds = lowrank_split(cfg_d, n_cp)
            lr[cfg_d.name.split("-")[0]] = (cfg_d, dd, spds)
    del keep_c5
    if "prefill" in sections:
        # (C2 also at a calibration-length batch: from 8192 tokens on its two middle products run as
        # one launch that never stores h2)
        for nm, cfg_d, dd, spds, Tp in [(nm, *v, v[0].prefill_T) for nm, v in lr.items()] + \
                                       [("C2", *lr["C2"], 16384)]:
            key = f"{nm}_prefill" if Tp == cfg_d.prefill_T else f"{nm}_prefill_T{Tp}"
            wsd = torch.empty(ff.workspace_bytes(dd, ff.WS_FORWARD, Tp), dtype=torch.uint8, device="cuda")
            xp = [torch.randn((Tp, cfg_d.d_model), device="cuda").to(bf) for _ in range(2)]
            yp = torch.empty((Tp, cfg_d.d_model), dtype=bf, device="cuda")
            st = {"i": 0}

            def pstep():
                ff.forward(dd, spds[st["i"] % len(spds)], xp[st["i"] & 1], yp, False, wsd)
                st["i"] += 1

            tpf, _ = timed(pstep, 200 if (cfg_d is C2 and Tp <= 4096) else 40, 10)
            flp = cfg_d.flops_per_token() * Tp
            note(f"{cfg_d.name} prefill T={Tp}: {tpf*1e6:.1f} us ({flp/tpf/1e12:.0f} TFLOP/s)")
            per[key] = {"workload": f"{cfg_d.name}: one ffsplit_forward, T={Tp}", "bound": "mfma",
                                    "achieved": flp / tpf / 1e12, "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
                                    "frac": flp / tpf / MFMA_BF16_PEAK, "traffic": traffic.get(key),
                                    "flops_per_launch": flp, "us_per_launch_hip_events": tpf * 1e6,
                                    "tokens_per_s": Tp / tpf}
            del wsd, xp, yp

    # ------------------------------------------------------------ bf16 low-rank decode (HBM-bound)
    if "decode" in sections:
        dl = {}
        for nm, (cfg_d, dd, spds) in lr.items():
            for B in cfg_d.decode_B:
                wsd = torch.empty(ff.workspace_bytes(dd, ff.WS_FORWARD, B), dtype=torch.uint8, device="cuda")
                xb = torch.randn((B, cfg_d.d_model), device="cuda").to(bf)
                yb = torch.empty((B, cfg_d.d_model), dtype=bf, device="cuda")
                st = {"i": 0}

                def lstep():
                    ff.forward(dd, spds[st["i"] % len(spds)], xb, yb, False, wsd)
                    st["i"] += 1

                td, _ = timed(lstep, 100, 20)
                note(f"{cfg_d.name} low-rank decode B={B}: {td*1e6:.1f} us")
                dl[f"{nm}_B{B}"] = {"us": td * 1e6, "tokens_per_s": B / td, "bytes_per_step": cfg_d.weight_bytes(),
                                    "GBps": cfg_d.weight_bytes() / td / 1e9, "frac_hbm": cfg_d.weight_bytes() / td / HBM_PEAK,
                                    "split_copies": len(spds)}
                per[f"{nm}_lowrank_decode_B{B}"] = {
                    "workload": f"{cfg_d.name}: one ffsplit_forward, batch {B}", "bound": "hbm",
                    "achieved": cfg_d.weight_bytes() / td / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                    "frac": cfg_d.weight_bytes() / td / HBM_PEAK, "traffic": traffic.get(f"{nm}_lowrank_decode"),
                    "bytes_per_launch": cfg_d.weight_bytes(), "us_per_launch_hip_events": td * 1e6, "tokens_per_s": B / td}
        out["decode_lowrank_bf16"] = {"workload": "C3 Llama-2-7B-shaped (k=550, rank 1024) and one C5 OPT-13B-shaped "
                                                  "layer (k=819, rank 1280): heavy bf16 + low-rank factors", **dl}
    del lr
    torch.cuda.empty_cache()

    # ------------------------------------------------------------ int4 decode (HBM-bound) and int4 prefill
    if "decode" in sections or "w3h8" in sections:
        c4 = C4
        L4 = device_layer(dataclasses.replace(c4, rank=8), 7004)     # (the factors are not used)
        Tp = 4096
        fl4 = 6.0 * Tp * c4.d_model * c4.d_ff          # the layer's dense products: a quantised split skips none
    if "decode" in sections:
        d4 = ff.make_desc(c4.d_model, c4.d_ff, c4.act, c4.dtype, c4.k, "int4", 0, c4.group)
        s4 = ff.build_split(d4, L4["W1"], L4["Wg"], L4["W2"], L4["idx"])
        torch.cuda.synchronize()
        n_copies = 16                                   # 16 x 80.8 MB = 1.3 GB >> 256 MB last-level cache
        s4s = [s4] + [s4.clone() for _ in range(n_copies - 1)]
        ws4 = torch.empty(ff.workspace_bytes(d4, ff.WS_FORWARD, 16), dtype=torch.uint8, device="cuda")
        dec = {}
        for B in c4.decode_B:
            xb = torch.randn((B, c4.d_model), device="cuda").to(bf)
            yb = torch.empty((B, c4.d_model), dtype=bf, device="cuda")
            st = {"i": 0}

            def dstep():
                ff.forward(d4, s4s[st["i"] % n_copies], xb, yb, False, ws4)
                st["i"] += 1

            t4, _ = timed(dstep, 160, 32)
            note(f"int4 decode B={B}: {t4*1e6:.1f} us ({c4.weight_bytes()/t4/1e9:.0f} GB/s)")
            dec[f"B{B}"] = {"us": t4 * 1e6, "tokens_per_s": B / t4, "GBps": c4.weight_bytes() / t4 / 1e9,
                            "frac_hbm": c4.weight_bytes() / t4 / HBM_PEAK}
            per[f"C4_int4_decode_B{B}"] = {"workload": f"{c4.name}: one ffsplit_forward, batch {B}", "bound": "hbm",
                                           "achieved": c4.weight_bytes() / t4 / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                                           "frac": c4.weight_bytes() / t4 / HBM_PEAK,
                                           "traffic": traffic.get(f"C4_int4_decode_B{B}"),
                                           "bytes_per_launch": c4.weight_bytes(), "us_per_launch_hip_events": t4 * 1e6,
                                           "tokens_per_s": B / t4}
        out["decode_int4"] = {"workload": "C4 Llama-2-7B-shaped SwiGLU, k=550 bf16 heavy + int4-g128 remainder",
                              "bytes_per_step": c4.weight_bytes(), "split_copies": n_copies, **dec}
        # the same split with many tokens: weights expanded to bf16 once per call, then dense MFMA products
        wsp = torch.empty(ff.workspace_bytes(d4, ff.WS_FORWARD, Tp), dtype=torch.uint8, device="cuda")
        xp = torch.randn((Tp, c4.d_model), device="cuda").to(bf)
        yp = torch.empty((Tp, c4.d_model), dtype=bf, device="cuda")
        tp4, _ = timed(lambda: ff.forward(d4, s4, xp, yp, False, wsp), 10, 3)
        note(f"int4 prefill T={Tp}: {tp4*1e6:.1f} us")
        out["prefill_int4"] = {"workload": f"C4 layer, T={Tp}", "us": tp4 * 1e6, "tokens_per_s": Tp / tp4,
                               "flops": fl4, "TFLOPs": fl4 / tp4 / 1e12, "frac_mfma": fl4 / tp4 / MFMA_BF16_PEAK}
        del wsp, xp, yp, s4s, s4, ws4
        torch.cuda.empty_cache()

    # ------------------------------------------------------------ 8-bit heavy / 3-bit remainder (Sec. 5.2's pairing)
    if "w3h8" in sections:
        d38 = ff.make_desc(c4.d_model, c4.d_ff, c4.act, c4.dtype, c4.k, "w3h8", 0, 128)
        s38 = ff.build_split(d38, L4["W1"], L4["Wg"], L4["W2"], L4["idx"])
        torch.cuda.synchronize()
        m4 = c4.d_ff - c4.k
        bytes38 = 3.0 * c4.k * c4.d_model + 3.0 * m4 * c4.d_model * 3 / 8 + 3.0 * c4.d_ff * (c4.d_model // 128) * 2
        n38 = 20                                        # 20 x 57.6 MB = 1.15 GB >> last-level cache
        s38s = [s38] + [s38.clone() for _ in range(n38 - 1)]
        ws38 = torch.empty(ff.workspace_bytes(d38, ff.WS_FORWARD, 32), dtype=torch.uint8, device="cuda")
        q38 = {}
        for B in c4.decode_B:
            xb = torch.randn((B, c4.d_model), device="cuda").to(bf)
            yb = torch.empty((B, c4.d_model), dtype=bf, device="cuda")
            st = {"i": 0}

            def qstep():
                ff.forward(d38, s38s[st["i"] % n38], xb, yb, False, ws38)
                st["i"] += 1

            t38, _ = timed(qstep, 100, 20)
            note(f"w3h8 decode B={B}: {t38*1e6:.1f} us")
            q38[f"B{B}"] = {"us": t38 * 1e6, "tokens_per_s": B / t38, "GBps": bytes38 / t38 / 1e9,
                            "frac_hbm": bytes38 / t38 / HBM_PEAK}
            per[f"C4_w3h8_decode_B{B}"] = {
                "workload": f"{c4.name} shape with int8 heavy / int3 remainder: one ffsplit_forward, batch {B}",
                "bound": "hbm", "achieved": bytes38 / t38 / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "frac": bytes38 / t38 / HBM_PEAK, "traffic": traffic.get("C4_w3h8_decode"),
                "bytes_per_launch": bytes38, "us_per_launch_hip_events": t38 * 1e6, "tokens_per_s": B / t38}
        wsp = torch.empty(ff.workspace_bytes(d38, ff.WS_FORWARD, Tp), dtype=torch.uint8, device="cuda")
        xp = torch.randn((Tp, c4.d_model), device="cuda").to(bf)
        yp = torch.empty((Tp, c4.d_model), dtype=bf, device="cuda")
        tp38, _ = timed(lambda: ff.forward(d38, s38, xp, yp, False, wsp), 10, 3)
        note(f"w3h8 prefill T={Tp}: {tp38*1e6:.1f} us")
        out["w3h8"] = {"workload": "C4 layer with Sec. 5.2's pairing: heavy int8-g128, remainder int3-g128",
                       "bytes_per_step": bytes38, "split_copies": n38, **q38,
                       "prefill_T4096": {"us": tp38 * 1e6, "tokens_per_s": Tp / tp38, "TFLOPs": fl4 / tp38 / 1e12,
                                         "frac_mfma": fl4 / tp38 / MFMA_BF16_PEAK}}
        del wsp, xp, yp, s38s, s38, ws38
    if "decode" in sections or "w3h8" in sections:
        del L4
        torch.cuda.empty_cache()

    # ------------------------------------------------------------ the calibration pipeline on the C2 layer
    if "pipeline" in sections:
        c2 = C2
        L2 = wl.make_layer(c2)
        W1, W2 = dev(L2["W1"]), dev(L2["W2"])
        Xc = dev(wl.make_tokens(c2, c2.calib_T, wl.gen.S_CALIB))
        d2 = ff.make_desc(c2.d_model, c2.d_ff, c2.act, c2.dtype, c2.k, "lowrank", c2.rank)
        acc = torch.zeros(2 * c2.d_ff, dtype=torch.float32, device="cuda")
        scores = torch.empty(c2.d_ff, dtype=torch.float32, device="cuda")
        ws_score = torch.empty(ff.workspace_bytes(d2, ff.WS_SCORE, c2.calib_T), dtype=torch.uint8, device="cuda")

        def do_score():
            acc.zero_()
            ff.score_neurons(d2, Xc, W1, None, W2, acc, 0, scores, ff.SCORE_SUMSQ, ws_score)

        t_score, _ = timed(do_score, 5, 2)
        t_select, _ = timed(lambda: ff.select_heavy(scores, c2.k), 5, 2)
        idx, _, flag = ff.select_heavy(scores, c2.k)
        torch.cuda.synchronize()
        ok2 = bool(np.array_equal(np.sort(idx.cpu().numpy()), L2["planted"])) and int(flag.item()) == 0
        ws_fact = torch.empty(ff.workspace_bytes(d2, ff.WS_FACTORIZE, 0), dtype=torch.uint8, device="cuda")
        t_fact, _ = timed(lambda: ff.factorize_remainder(d2, W1, None, W2, idx, 1, ws_fact), 2, 1)
        facd = ff.factorize_remainder(d2, W1, None, W2, idx, 1, ws_fact)
        sp2 = ff.build_split(d2, W1, None, W2, idx, facd)
        t_build, _ = timed(lambda: ff.build_split(d2, W1, None, W2, idx, facd, sp2), 3, 1)
        note(f"C2 pipeline: score {t_score*1e6:.0f} us, select {t_select*1e6:.0f} us, factorise {t_fact*1e3:.1f} ms, "
             f"build {t_build*1e6:.0f} us, heavy set ok={ok2}")
        out["pipeline"] = {"workload": "C2 layer: score (4096 tokens) -> select -> factorise on the device -> build",
                           "score_us_T4096": t_score * 1e6,
                           "score_tflops": 2.0 * c2.calib_T * c2.d_model * c2.d_ff / t_score / 1e12,
                           "select_us": t_select * 1e6, "build_split_us": t_build * 1e6,
                           "factorize_on_device_ms": t_fact * 1e3, "heavy_set_equals_planted": ok2}
        del W1, W2, Xc, ws_score, ws_fact, facd, sp2
        torch.cuda.empty_cache()

    # ------------------------------------------------------------ C1, the fp32 correctness config
    if "c1" in sections:
        c1 = C1
        L1 = wl.make_layer(c1)
        f1 = wl.make_factors(c1, L1, L1["planted"])
        f32 = torch.float32
        d1 = ff.make_desc(c1.d_model, c1.d_ff, c1.act, c1.dtype, c1.k, "lowrank", c1.rank)
        s1 = ff.build_split(d1, dev(L1["W1"], f32), None, dev(L1["W2"], f32), torch.from_numpy(L1["planted"]).cuda(),
                            {k: dev(v, f32) for k, v in f1.items()})
        x1 = dev(wl.make_tokens(c1, c1.prefill_T), f32)
        y1 = torch.empty((c1.prefill_T, c1.d_model), dtype=f32, device="cuda")
        w1s = torch.empty(ff.workspace_bytes(d1, ff.WS_FORWARD, c1.prefill_T), dtype=torch.uint8, device="cuda")
        t1, _ = timed(lambda: ff.forward(d1, s1, x1, y1, False, w1s), 100, 20)
        note(f"C1 fp32 forward T={c1.prefill_T}: {t1*1e6:.1f} us")
        out["c1_fp32"] = {"workload": "C1 BERT-base-shaped layer, fp32, T=128 (correctness config; launch-latency bound)",
                          "us": t1 * 1e6, "tokens_per_s": c1.prefill_T / t1,
                          "GFLOPs": c1.flops_per_token() * c1.prefill_T / t1 / 1e9}

    # ------------------------------------------------------------ measured ceilings of this machine
    # The library's own probe kernels (csrc/probe.hip): a pure matrix-core loop and a streaming read,
    # auditable denominators next to the datasheet peaks the fractions above are quoted against.
    if "yardsticks" in sections:
        torch.cuda.empty_cache()
        scr = torch.zeros(64, dtype=torch.uint8, device="cuda")
        fl = {"v": 0.0}

        def mf():
            fl["v"] = ff.probe_mfma(2048, 4096, scr)

        tm, _ = timed(mf, 10, 2)
        chunk = 80 << 20
        bufs = torch.empty(16 * chunk, dtype=torch.uint8, device="cuda")
        bufs.fill_(1)
        st = {"i": 0}

        def rd():
            i = st["i"] % 16
            ff.probe_stream_read(bufs[i * chunk:(i + 1) * chunk], 2048, scr)
            st["i"] += 1

        tr, _ = timed(rd, 64, 16)
        def stream_floor(sizes, reps=20):
            """us per pass of a sequence of plain streaming-read launches of the given byte counts,
            replayed from a HIP graph (no host time between the launches): what the same bytes in the
            same number of dependent launches cost with no arithmetic at all."""
            views, o = [], 0
            for _ in range(reps):
                for nb in sizes:
                    nb = int(nb) // 4096 * 4096
                    if o + nb > bufs.numel():
                        o = 0
                    views.append(bufs[o:o + nb])
                    o += nb
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for v in views[:len(sizes)]:
                    ff.probe_stream_read(v, 2048, scr)
                side.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    for v in views:
                        ff.probe_stream_read(v, 2048, scr)
            torch.cuda.synchronize()
            tg, _ = timed(g.replay, 10, 3)
            return tg / reps * 1e6

        MBs = 1e6
        c3w, c4w, c5w = C3.weight_bytes(), C4.weight_bytes(), C5.weight_bytes()

        def lowrank_launch_bytes(c):
            nu = 2 if c.act == "swiglu" else 1
            m = c.d_ff - c.k
            g = [2 * c.d_model * nu * (c.k + c.rank), 2 * nu * c.rank * m, 2 * m * c.rank, 2 * (c.k + c.rank) * c.d_model]
            # G1 and G3 are a streaming launch plus a summing launch that reads a few MB of partials
            return [g[0], 4 * MBs, g[1], g[2], 4 * MBs, g[3]]

        floors = {
            "C4_int4_decode (2 launches: up/gate 2/3 of the bytes, down 1/3)": stream_floor([c4w * 2 / 3, c4w / 3]),
            "C3_lowrank_decode (6 launches)": stream_floor(lowrank_launch_bytes(C3)),
            "C5_lowrank_decode (6 launches)": stream_floor(lowrank_launch_bytes(C5)),
            "C4_w3h8_decode (4 launches: 38 MB, 4 MB of partials, 19 MB, 4 MB)": stream_floor([38 * MBs, 4 * MBs, 19 * MBs, 4 * MBs]),
            "one launch of 1 MB (fixed cost of a dependent launch)": stream_floor([1 * MBs]),
        }
        note("streaming-read floors of the decode launch sequences (us): " +
             ", ".join(f"{k.split(' ')[0]} {v:.1f}" for k, v in floors.items()))
        out["yardsticks"] = {"pure_mfma_loop_TFLOPs": fl["v"] / tm / 1e12,
                             "decode_launch_sequence_stream_floor_us": floors,
                             "streaming_read_80MB_GBps": chunk / tr / 1e9, "streaming_read_80MB_us": tr * 1e6,
                             "note": "ffsplit_probe_mfma / ffsplit_probe_stream_read: this library's own kernels, "
                                     "measurement only, rotating over 16 x 80 MB for the read"}
        note(f"ceilings: pure MFMA loop {fl['v']/tm/1e12:.0f} TFLOP/s, streaming read of 80 MB {tr*1e6:.1f} us "
             f"({chunk/tr/1e9:.0f} GB/s)")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
