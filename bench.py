#!/usr/bin/env python3
"""Benchmark of the split feed-forward layer on one MI355X.

Headline workload: the OPT-1.3B-shaped layer (d_model 2048, d_ff 8192, GeLU,
bf16, k = 246 heavy neurons, rank-512 remainder), prefill of 8 x 512 = 4096
tokens.  A step is one ffsplit_forward over that batch; the split it runs on
comes from the library's own score -> select -> build calls (timed once, reported
under "pipeline").  Inputs, weights and the packed split are resident in HBM
before the timed region.  Prints ONE JSON line.

Also measured, as extra keys, against the HBM roofline (rotating over enough
split copies that every weight byte comes from HBM, not from the 256 MB
last-level cache): the int4 decode of the Llama-2-7B-shaped layer at batch
1/4/16, and the bf16 low-rank decode of the Llama-2-7B-shaped layer (batch
1/8/32) and of one OPT-13B-shaped layer (batch 16).
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
# HBM bytes of one C2 forward (read + written), from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/gemm_bf16_chain_C2_prefill.md (scaled by the reference copy there)
TRAFFIC_C2_PREFILL = 379.5e6   # 269.9 MB read + 109.6 MB written


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-decode", action="store_true", help="skip the decode sections")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-yardsticks", action="store_true",
                    help="skip the machine yardsticks (device copy, vendor-library GEMMs through torch)")
    ap.add_argument("--preheat-ms", type=float, default=100.0,
                    help="untimed steady load before every timed loop, so that the clocks have settled")
    ap.add_argument("--copies", type=int, default=4, help="split copies rotated through in the prefill loop")
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

    def note(msg):
        print(f"[bench {time.perf_counter() - t_start:6.1f}s] {msg}", file=sys.stderr, flush=True)

    def dev(a, dt=bf):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, np.float32)).to("cuda", dtype=dt)

    def timed(fn, n, warm):
        preheat_s = args.preheat_ms * 1e-3
        # The GPU's clocks take tens of milliseconds of continuous load to settle after the host-side
        # preparation that precedes every section (measured: the first ~10 ms of a loop run 5-15 %
        # slower than its steady state).  Untimed calls of the same step until preheat_s has passed,
        # then the warm-up steps asked for, then the timed ones.
        t_pre = time.perf_counter()
        while time.perf_counter() - t_pre < preheat_s:
            for _ in range(8):
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

    if args.calib_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        note("reference copy done: 3 x 256 MiB read + 256 MiB written")

    # ------------------------------------------------------------ headline: C2 prefill
    cfg = C2
    T = cfg.prefill_T
    L = wl.make_layer(cfg)
    note("C2 weights generated")
    W1, W2 = dev(L["W1"]), dev(L["W2"])
    Xc = dev(wl.make_tokens(cfg, cfg.calib_T, wl.gen.S_CALIB))
    desc = ff.make_desc(cfg.d_model, cfg.d_ff, cfg.act, cfg.dtype, cfg.k, "lowrank", cfg.rank)
    acc = torch.zeros(2 * cfg.d_ff, dtype=torch.float32, device="cuda")
    scores = torch.empty(cfg.d_ff, dtype=torch.float32, device="cuda")
    ws_score = torch.empty(ff.workspace_bytes(desc, ff.WS_SCORE, cfg.calib_T), dtype=torch.uint8, device="cuda")

    def do_score():
        acc.zero_()
        ff.score_neurons(desc, Xc, W1, None, W2, acc, 0, scores, ff.SCORE_SUMSQ, ws_score)

    t_score, _ = timed(do_score, 5, 2)
    t_select, _ = timed(lambda: ff.select_heavy(scores, cfg.k), 5, 2)
    idx, _, flag = ff.select_heavy(scores, cfg.k)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    heavy_ok = bool(np.array_equal(np.sort(idx_h), L["planted"])) and int(flag.item()) == 0
    note(f"score {t_score*1e6:.0f} us, select {t_select*1e6:.0f} us, heavy set ok={heavy_ok}")
    fac = wl.make_factors(cfg, L, idx_h)
    note("rank-512 factors of the remainder computed (host)")
    facd = {k: dev(v) for k, v in fac.items()}
    split0 = ff.build_split(desc, W1, None, W2, idx, facd)
    t_build, _ = timed(lambda: ff.build_split(desc, W1, None, W2, idx, facd, split0), 3, 1)
    ws_fact = torch.empty(ff.workspace_bytes(desc, ff.WS_FACTORIZE, 0), dtype=torch.uint8, device="cuda")
    t_fact, _ = timed(lambda: ff.factorize_remainder(desc, W1, None, W2, idx, 1, ws_fact), 2, 1)
    del ws_fact
    splits = [split0] + [split0.clone() for _ in range(max(args.copies, 1) - 1)]
    Xe_h = wl.make_tokens(cfg, T)
    Xs = [dev(Xe_h)] + [dev(wl.make_tokens(cfg, T, wl.gen.S_EVAL, layer=i)) for i in range(1, len(splits))]
    Y = torch.empty((T, cfg.d_model), dtype=bf, device="cuda")
    ws = torch.empty(ff.workspace_bytes(desc, ff.WS_FORWARD, T), dtype=torch.uint8, device="cuda")
    del Xc, ws_score
    state = {"i": 0}

    def step():
        i = state["i"] % len(splits)
        state["i"] += 1
        ff.forward(desc, splits[i], Xs[i], Y, False, ws)

    t_ev, t_wall = timed(step, args.steps, args.warmup)
    flops = cfg.flops_per_token() * T
    note(f"forward {t_ev*1e6:.1f} us/step (events), {t_wall*1e6:.1f} us/step (wall)")
    # parity of the timed configuration on sampled rows (rows of X are independent)
    from oracle import ffsplit_oracle as orc
    ff.forward(desc, splits[0], Xs[0], Y, False, ws)
    torch.cuda.synchronize()
    rows = np.random.default_rng(0).choice(T, 32, replace=False)
    want = orc.forward_split(Xe_h[rows], L["W1"], L["W2"], None, idx_h, "gelu", "lowrank", fac)[0]
    got = Y[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
    rel_err = float(np.linalg.norm(got - want) / np.linalg.norm(want))

    out = {
        "metric": "split-FFN tokens/s per layer; % of MFMA peak (prefill) / HBM BW (decode)",
        "value": T / t_wall,
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
        "config": {"workload": "C2 OPT-1.3B-shaped split FFN prefill: d_model=2048 d_ff=8192 GeLU k=246 rank=512 "
                               "T=8x512=4096, one layer", "split_copies": len(splits),
                   "preheat_ms": args.preheat_ms},
        "roofline": {"bound": "mfma",
                     "kernel": "ffsplit_forward = 4 chained gemm_bf16_dl_kernel launches (+ split-K sum); "
                               "per-launch figures in profiles/",
                     "achieved": flops / t_ev / 1e12, "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
                     "frac": flops / t_ev / MFMA_BF16_PEAK, "traffic": TRAFFIC_C2_PREFILL,
                     "flops_per_launch": flops, "us_per_launch_hip_events": t_ev * 1e6},
        "parity": {"rel_frobenius_vs_oracle_32_rows": rel_err, "heavy_set_equals_planted": heavy_ok},
        "pipeline": {"score_us_T4096": t_score * 1e6,
                     "score_tflops": 2.0 * cfg.calib_T * cfg.d_model * cfg.d_ff / t_score / 1e12,
                     "select_us": t_select * 1e6, "build_split_us": t_build * 1e6,
                     "factorize_on_device_ms": t_fact * 1e3},
    }

    # ------------------------------------------------------------ cpu baseline: the oracle as it stands
    if not args.no_cpu:
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        reps, spent = 0, 0.0
        while spent < 10.0 and reps < 8:
            t0 = time.perf_counter()
            orc.forward_split(Xe_h, L["W1"], L["W2"], None, idx_h, "gelu", "lowrank", fac)
            spent += time.perf_counter() - t0
            reps += 1
        note(f"oracle timed: {reps} reps in {spent:.1f} s")
        out["cpu_baseline"] = {"value": T * reps / spent, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{reps} x the full {T}-token forward of the same layer (numpy fp64)"}

    # ------------------------------------------------------------ extra: int4 decode (HBM-bound)
    if not args.no_decode:
        del splits, Xs, W1, W2, facd
        torch.cuda.empty_cache()
        c4 = C4
        L4 = wl.make_layer(c4)
        note("C4 weights generated")
        d4 = ff.make_desc(c4.d_model, c4.d_ff, c4.act, c4.dtype, c4.k, "int4", 0, c4.group)
        s4 = ff.build_split(d4, dev(L4["W1"]), dev(L4["Wg"]), dev(L4["W2"]), torch.from_numpy(L4["planted"]).cuda())
        torch.cuda.synchronize()
        n_copies = 16                                   # 16 x 80.8 MB = 1.3 GB >> 256 MB last-level cache
        s4s = [s4] + [s4.clone() for _ in range(n_copies - 1)]
        ws4 = torch.empty(ff.workspace_bytes(d4, ff.WS_FORWARD, 16), dtype=torch.uint8, device="cuda")
        dec = {}
        for B in c4.decode_B:
            xb = dev(wl.make_tokens(c4, B))
            yb = torch.empty((B, c4.d_model), dtype=bf, device="cuda")
            st = {"i": 0}

            def dstep():
                ff.forward(d4, s4s[st["i"] % n_copies], xb, yb, False, ws4)
                st["i"] += 1

            t4, _ = timed(dstep, 160, 32)
            note(f"int4 decode B={B}: {t4*1e6:.1f} us")
            dec[f"B{B}"] = {"us": t4 * 1e6, "tokens_per_s": B / t4, "GBps": c4.weight_bytes() / t4 / 1e9,
                            "frac_hbm": c4.weight_bytes() / t4 / HBM_PEAK}
        out["decode_int4"] = {"workload": "C4 Llama-2-7B-shaped SwiGLU, k=550 bf16 heavy + int4-g128 remainder",
                              "bytes_per_step": c4.weight_bytes(), "split_copies": n_copies, **dec}
        # the same split with many tokens: weights expanded to bf16 once per call, then dense MFMA products
        Tp = 4096
        wsp = torch.empty(ff.workspace_bytes(d4, ff.WS_FORWARD, Tp), dtype=torch.uint8, device="cuda")
        xp = dev(wl.make_tokens(c4, Tp))
        yp = torch.empty((Tp, c4.d_model), dtype=bf, device="cuda")
        tp4, _ = timed(lambda: ff.forward(d4, s4, xp, yp, False, wsp), 10, 3)
        fl4 = 6.0 * Tp * c4.d_model * c4.d_ff          # the layer's dense products: the int4 split skips none
        note(f"int4 prefill T={Tp}: {tp4*1e6:.1f} us")
        out["prefill_int4"] = {"workload": f"C4 layer, T={Tp}", "us": tp4 * 1e6, "tokens_per_s": Tp / tp4,
                               "flops": fl4, "TFLOPs": fl4 / tp4 / 1e12, "frac_mfma": fl4 / tp4 / MFMA_BF16_PEAK}
        del wsp, xp, yp, s4s, s4, ws4
        torch.cuda.empty_cache()

        # ------------------------------------------------------------ extra: 8-bit heavy / 3-bit remainder
        d38 = ff.make_desc(c4.d_model, c4.d_ff, c4.act, c4.dtype, c4.k, "w3h8", 0, 128)
        s38 = ff.build_split(d38, dev(L4["W1"]), dev(L4["Wg"]), dev(L4["W2"]), torch.from_numpy(L4["planted"]).cuda())
        torch.cuda.synchronize()
        m4 = c4.d_ff - c4.k
        bytes38 = 3.0 * c4.k * c4.d_model + 3.0 * m4 * c4.d_model * 3 / 8 + 3.0 * c4.d_ff * (c4.d_model // 128) * 2
        n38 = 20                                        # 20 x 57.6 MB = 1.15 GB >> last-level cache
        s38s = [s38] + [s38.clone() for _ in range(n38 - 1)]
        ws38 = torch.empty(ff.workspace_bytes(d38, ff.WS_FORWARD, 32), dtype=torch.uint8, device="cuda")
        q38 = {}
        for B in c4.decode_B:
            xb = dev(wl.make_tokens(c4, B))
            yb = torch.empty((B, c4.d_model), dtype=bf, device="cuda")
            st = {"i": 0}

            def qstep():
                ff.forward(d38, s38s[st["i"] % n38], xb, yb, False, ws38)
                st["i"] += 1

            t38, _ = timed(qstep, 100, 20)
            note(f"w3h8 decode B={B}: {t38*1e6:.1f} us")
            q38[f"B{B}"] = {"us": t38 * 1e6, "tokens_per_s": B / t38, "GBps": bytes38 / t38 / 1e9,
                            "frac_hbm": bytes38 / t38 / HBM_PEAK}
        wsp = torch.empty(ff.workspace_bytes(d38, ff.WS_FORWARD, Tp), dtype=torch.uint8, device="cuda")
        xp = dev(wl.make_tokens(c4, Tp))
        yp = torch.empty((Tp, c4.d_model), dtype=bf, device="cuda")
        tp38, _ = timed(lambda: ff.forward(d38, s38, xp, yp, False, wsp), 10, 3)
        note(f"w3h8 prefill T={Tp}: {tp38*1e6:.1f} us")
        out["w3h8"] = {"workload": "C4 layer with Sec. 5.2's pairing: heavy int8-g128, remainder int3-g128",
                       "bytes_per_step": bytes38, "split_copies": n38, **q38,
                       "prefill_T4096": {"us": tp38 * 1e6, "tokens_per_s": Tp / tp38, "TFLOPs": fl4 / tp38 / 1e12,
                                         "frac_mfma": fl4 / tp38 / MFMA_BF16_PEAK}}
        del wsp, xp, yp, s38s, s38, ws38


        # ------------------------------------------------------------ extra: bf16 low-rank decode (HBM-bound)
        torch.cuda.empty_cache()
        dl, pl = {}, {}
        for cfg_d, n_cp in ((C3, 10), (C5, 8)):
            Ld = wl.make_layer(cfg_d)
            facs = wl.make_factors(dataclasses.replace(cfg_d, exact_svd=False), Ld, Ld["planted"])
            dd = ff.make_desc(cfg_d.d_model, cfg_d.d_ff, cfg_d.act, cfg_d.dtype, cfg_d.k, "lowrank", cfg_d.rank)
            spd = ff.build_split(dd, dev(Ld["W1"]), dev(Ld["Wg"]), dev(Ld["W2"]),
                                 torch.from_numpy(Ld["planted"]).cuda(), {k: dev(v) for k, v in facs.items()})
            torch.cuda.synchronize()
            spds = [spd] + [spd.clone() for _ in range(n_cp - 1)]
            note(f"{cfg_d.name}: split built, {n_cp} copies of {cfg_d.weight_bytes()/1e6:.0f} MB")
            for B in cfg_d.decode_B:
                wsd = torch.empty(ff.workspace_bytes(dd, ff.WS_FORWARD, B), dtype=torch.uint8, device="cuda")
                xb = dev(wl.make_tokens(cfg_d, B))
                yb = torch.empty((B, cfg_d.d_model), dtype=bf, device="cuda")
                st = {"i": 0}

                def lstep():
                    ff.forward(dd, spds[st["i"] % n_cp], xb, yb, False, wsd)
                    st["i"] += 1

                td, _ = timed(lstep, 100, 20)
                note(f"{cfg_d.name} low-rank decode B={B}: {td*1e6:.1f} us")
                dl[f"{cfg_d.name.split('-')[0]}_B{B}"] = {
                    "us": td * 1e6, "tokens_per_s": B / td, "bytes_per_step": cfg_d.weight_bytes(),
                    "GBps": cfg_d.weight_bytes() / td / 1e9, "frac_hbm": cfg_d.weight_bytes() / td / HBM_PEAK}
            # prefill of the same layer (MFMA-bound)
            Tp = cfg_d.prefill_T
            wsd = torch.empty(ff.workspace_bytes(dd, ff.WS_FORWARD, Tp), dtype=torch.uint8, device="cuda")
            xp = dev(wl.make_tokens(cfg_d, Tp))
            yp = torch.empty((Tp, cfg_d.d_model), dtype=bf, device="cuda")
            st = {"i": 0}

            def pstep():
                ff.forward(dd, spds[st["i"] % n_cp], xp, yp, False, wsd)
                st["i"] += 1

            tpf, _ = timed(pstep, 20, 5)
            flp = cfg_d.flops_per_token() * Tp
            note(f"{cfg_d.name} prefill T={Tp}: {tpf*1e6:.1f} us")
            pl[cfg_d.name.split('-')[0]] = {"T": Tp, "us": tpf * 1e6, "tokens_per_s": Tp / tpf, "flops": flp,
                                            "TFLOPs": flp / tpf / 1e12, "frac_mfma": flp / tpf / MFMA_BF16_PEAK}
            del spds, spd, wsd, xp, yp
            torch.cuda.empty_cache()
        out["prefill_lowrank_bf16"] = {"workload": "the same C3 and C5 layers, 4096 tokens", **pl}
        out["decode_lowrank_bf16"] = {"workload": "C3 Llama-2-7B-shaped (k=550, rank 1024) and one C5 OPT-13B-shaped "
                                                  "layer (k=819, rank 1280): heavy bf16 + low-rank factors, seeded "
                                                  "Gaussian factors", **dl}

    # ------------------------------------------------------------ extra: C1, the fp32 correctness config
    if not args.no_decode:
        torch.cuda.empty_cache()
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

    # ------------------------------------------------------------ yardsticks of this machine (not the product path)
    # What the same box gives to a plain device copy and to the vendor BLAS behind torch.matmul:
    # auditable denominators next to the datasheet peaks the fractions above are quoted against.
    if not args.no_yardsticks:
        torch.cuda.empty_cache()
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        tc, _ = timed(lambda: dst.copy_(src), 10, 3)
        del src, dst
        a8 = torch.randn(8192, 8192, dtype=bf, device="cuda")
        b8 = torch.randn(8192, 8192, dtype=bf, device="cuda")
        tg, _ = timed(lambda: torch.matmul(a8, b8), 10, 3)
        del a8, b8
        # the four products of the C2 chain as plain library GEMMs plus a separate GeLU pass
        c2 = C2
        Tq, dq, kq, rq = c2.prefill_T, c2.d_model, c2.k, c2.rank
        mq = c2.d_ff - kq
        xq = torch.randn(Tq, dq, dtype=bf, device="cuda")
        w1q = torch.randn(dq, kq + rq, dtype=bf, device="cuda")
        q1q = torch.randn(rq, mq, dtype=bf, device="cuda")
        p2q = torch.randn(mq, rq, dtype=bf, device="cuda")
        w4q = torch.randn(kq + rq, dq, dtype=bf, device="cuda")

        def lib_chain():
            z = torch.matmul(xq, w1q)
            h = torch.nn.functional.gelu(torch.matmul(z[:, kq:], q1q))
            t2 = torch.matmul(h, p2q)
            return torch.matmul(torch.cat([torch.nn.functional.gelu(z[:, :kq]), t2], dim=1), w4q)

        tl, _ = timed(lib_chain, 20, 5)
        out["yardsticks"] = {"device_copy_1GiB_GBps_read_plus_write": 2.0 * (1 << 30) / tc / 1e9,
                             "torch_matmul_bf16_8192_TFLOPs": 2.0 * 8192 ** 3 / tg / 1e12,
                             "c2_chain_as_torch_ops_us": tl * 1e6,
                             "note": "vendor library / torch kernels, measurement only; not used by the product path"}
        note(f"yardsticks: copy {out['yardsticks']['device_copy_1GiB_GBps_read_plus_write']:.0f} GB/s, "
             f"matmul 8192^3 {out['yardsticks']['torch_matmul_bf16_8192_TFLOPs']:.0f} TFLOP/s, "
             f"C2 chain as torch ops {tl*1e6:.0f} us")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
