"""Summarise rocprofv3 output of bench.py into the short tables kept under profiles/.

    python -m paper_2401_04044_amd.profile_summary --kt DIR [--fetch DIR --write DIR] [--pmc DIR] --out profiles

DIR are rocprofv3 output directories (CSV output format):
  --kt     a `--kernel-trace` run of `bench.py` (every section);
  --fetch  a `--pmc FETCH_SIZE` run and --write a `--pmc WRITE_SIZE` run of `bench.py --calib-copy`
           (the 256 MiB reference copy scales the counters: KiB reported per KiB really moved);
  --pmc    a `--pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE
           SQ_WAIT_INST_LDS SQ_ACTIVE_INST_ANY` run.
Writes <out>/<workload>.md per workload and <out>/hbm_traffic.json (bytes per launch of each
workload, which bench.py reports as roofline.traffic).

A workload's launches are told apart by (kernel name pattern, workgroups): the same kernel
template serves several products.  The signature table below lists them as bench.py launches
them at the five workload shapes.
"""
import argparse
import collections
import csv
import glob
import json
import os
import re

# (label, kernel-name regex, workgroups x, workgroups y [, regex of the kernel launched just before])
# per workload: where two products share template and workgroup count, the chain's order tells them apart
G = r"gemm_bf16_dl_kernel<"
SIGNATURES = {
    "C5_stack_layer": [
        ("pre-norm  token_rmsnorm_kernel", r"token_rmsnorm_kernel<true>", 4096, 1),
        ("G1 X [W1h | P1]  128x320 tiles", G + r"128, 320, 32, 2, 2, 1, 3, 1, false, false, false, false>", 224, 1),
        ("G2 gelu(t Q1)  256x256 tiles", G + r"256, 256, 32, 2, 4, 1, 3, 1, false, false, true, false>", 1232, 1),
        ("G3 h2 P2  256x320 tiles x 4 splits", G + r"256, 320, 32, 4, 2, 1, 3, 0, false, false, true, false>", 64, 4, G),
        ("G3 sum of the splits", r"splitk_reduce_kernel", 2560, 1),
        ("G4 [h1 | t2] [W2h ; Q2] + residual, fp32 out  256x320 tiles", G + r"256, 320, 32, 4, 2, 1, 3, 0, false, false, true, true>", 256, 1),
    ],
    "C5_prefill": [
        ("G1  128x320 tiles", G + r"128, 320, 32, 2, 2, 1, 3, 1, false, false, false, false>", 224, 1),
        ("G2  256x256 tiles", G + r"256, 256, 32, 2, 4, 1, 3, 1, false, false, true, false>", 1232, 1),
        ("G3  256x320 tiles x 4 splits", G + r"256, 320, 32, 4, 2, 1, 3, 0, false, false, true, false>", 64, 4, G),
        ("G3 sum of the splits", r"splitk_reduce_kernel", 2560, 1),
        ("G4  256x320 tiles", G + r"256, 320, 32, 4, 2, 1, 3, 0, false, false, true, false>", 256, 1, r"splitk_reduce_kernel"),
    ],
    "C3_prefill": [
        ("G1 X [gate/up heavy | Pg | P1]  256x256 tiles", G + r"256, 256, 32, 2, 4, 1, 3, 2, false, false, false, false>", 208, 1),
        ("G2 silu(tg Qg) * (tu Q1), two left operands  256x256 tiles", G + r"256, 256, 32, 4, 2, 1, 3, 2, true, false, true, false>", 1312, 1),
        ("G3 h2 P2  256x256 tiles x 4 splits", G + r"256, 256, 32, 2, 4, 1, 3, 0, false, false, true, false>", 64, 4, G),
        ("G3 sum of the splits", r"splitk_reduce_kernel", 2048, 1),
        ("G4  256x256 tiles", G + r"256, 256, 32, 2, 4, 1, 3, 0, false, false, true, false>", 256, 1, r"splitk_reduce_kernel"),
    ],
    "C2_prefill": [
        ("G1  128x128 tiles, in-workgroup K split", G + r"128, 128, 64, 2, 2, 2, 4, 1, false, false, false, false>", 192, 1),
        ("G2  256x128 tiles", G + r"256, 128, 32, 2, 2, 1, 3, 1, false, false, true, false>", 1008, 1),
        ("G3  128x128 tiles, K split 2 x 2", G + r"128, 128, 64, 2, 2, 2, 4, 0, false, false, true, false>", 128, 2),
        ("G3 sum of the splits", r"splitk_reduce_kernel", 1024, 1),
        ("G4  128x128 tiles", G + r"128, 128, 32, 2, 2, 1, 3, 0, false, false, true, false>", 512, 1),
    ],
    "C2_prefill_T16384": [
        ("G1  256x256 tiles", G + r"256, 256, 32, 2, 4, 1, 3, 1, false, false, false, false>", 192, 1),
        ("G2 + G3 in one launch, h2 never stored: 128 rows x 2 neuron ranges", r"ffn2_fused_kernel", 256, 1),
        ("sum of the ranges", r"splitk_reduce_kernel", 4096, 1),
        ("G4  256x256 tiles", G + r"256, 256, 32, 2, 4, 1, 3, 0, false, false, true, false>", 512, 1),
    ],
    "C4_int4_decode": [
        ("phase 1: gate/up, activation", r"int4_phase1_kernel<4, 8, 2>", 253, 1),
        ("phase 2: down, sum", r"int4_phase2_kernel", 32, 8),
    ],
    "C4_int4_prefill": [
        ("expand up/gate to bf16", r"expand_up_kernel", 44288, 1),
        ("expand down to bf16", r"expand_down_kernel", 22144, 1),
        ("G1 X [W1 ; Wg]  256x256 tiles", G + r"256, 256, 32, 2, 4, 1, 3, 2, false, false, false, false>", 1392, 1),
        ("G4 h W2  256x256 tiles", G + r"256, 256, 32, 2, 4, 1, 3, 0, false, false, true, false>", 256, 1, G + r"256, 256, 32, 2, 4, 1, 3, 2,"),
    ],
    "C4_w3h8_decode": [
        ("up/gate stream (int8 heavy + int3 rest)", r"skinny_stream_q2_kernel<false>", 764, 1),
        ("sum, activation", r"skinny_reduce_kernel", 692, 1),
        ("down stream", r"skinny_stream_q2_kernel<true>", 576, 1),
        ("sum", r"skinny_reduce_kernel", 128, 1),
    ],
    "C3_lowrank_decode": [
        ("G1 stream", r"skinny_stream_kernel<false, 1>", 200, 1),
        ("G1 sum, activation", r"skinny_reduce_kernel", 100, 1),
        ("G2 (two left operands, SwiGLU)", r"skinny_fused_kernel<true, 2, 4, true>", 328, 1),
        ("G3 stream", r"skinny_stream_kernel<true, 1>", 160, 1),
        ("G3 sum", r"skinny_reduce_kernel", 32, 1),
        ("G4", r"skinny_fused_kernel<true, 1, 8, false>", 128, 1),
    ],
    "C5_lowrank_decode": [
        ("G1 stream", r"skinny_stream_kernel<false, 1>", 165, 1),
        ("G1 sum, activation", r"skinny_reduce_kernel", 66, 1),
        ("G2", r"skinny_fused_kernel<true, 2, 4, false>", 308, 1),
        ("G3 stream", r"skinny_stream_kernel<true, 1>", 250, 1),
        ("G3 sum", r"skinny_reduce_kernel", 40, 1),
        ("G4", r"skinny_fused_kernel<true, 1, 8, false>", 160, 1),
    ],
    "C2_calibration": [
        ("re-tile W1 (neuron-major)", r"permute_transpose_kernel<unsigned short>", 256, 64),
        ("score product X W1, gelu, column sums  256x256 tiles", G + r"256, 256, 32, 2, 4, 1, 3, 1, false, true, false, false>", 512, 1),
        ("sum of the row tiles' partials", r"reduce_partials_kernel", 32, 1),
        ("row norms of W2, score", r"finalize_scores_kernel<true>", 2048, 1),
        ("selection: bit search + compaction", r"select_compact_kernel<8>", 1, 1),
        ("selection: ranking", r"select_rank_kernel", 62, 1),
    ],
    "ceilings": [
        ("pure MFMA loop (ffsplit_probe_mfma)", r"probe_mfma_kernel", 2048, 1),
        ("streaming read of 80 MB (ffsplit_probe_stream_read)", r"probe_read_kernel", 2048, 1),
    ],
}
# workloads whose summed FETCH + WRITE bytes bench.py reports as roofline.traffic
TRAFFIC_KEYS = {"C5_stack_layer": "C5_stack_layer", "C5_prefill": "C5_prefill", "C3_prefill": "C3_prefill",
                "C2_prefill": "C2_prefill", "C2_prefill_T16384": "C2_prefill_T16384", "C4_int4_decode": ["C4_int4_decode_B1", "C4_int4_decode_B4",
                                                                "C4_int4_decode_B16"],
                "C3_lowrank_decode": "C3_lowrank_decode", "C5_lowrank_decode": "C5_lowrank_decode",
                "C4_w3h8_decode": "C4_w3h8_decode"}


def _short(name):
    name = name.replace("ffsplit::", "").replace("(anonymous namespace)::", "").replace("void ", "")
    return name


def _find(d, suffix):
    hits = sorted(glob.glob(os.path.join(d, "*" + suffix)))
    if not hits:
        raise FileNotFoundError(f"no *{suffix} in {d}")
    return hits[0]


class Dispatch:
    __slots__ = ("name", "gx", "gy", "wgs", "us", "counters", "prev")

    def __init__(self, name, gx, gy, wgs, us):
        self.name, self.gx, self.gy, self.wgs, self.us = name, gx, gy, wgs, us
        self.counters = {}
        self.prev = ""


def _chain(ds):
    """Dispatches in launch order, each with the name of the one before it."""
    ds = [d for _, d in sorted(ds.items())]
    for a, b in zip(ds, ds[1:]):
        b.prev = a.name
    return ds


def load_trace(d):
    ds = {}
    for r in csv.DictReader(open(_find(d, "kernel_trace.csv"))):
        gx = int(r["Grid_Size_X"]) // max(int(r["Workgroup_Size_X"]), 1)
        gy = int(r["Grid_Size_Y"]) // max(int(r["Workgroup_Size_Y"]), 1)
        ds[int(r["Dispatch_Id"])] = Dispatch(_short(r["Kernel_Name"]), gx, gy, gx * gy,
                                             (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    return _chain(ds)


def load_counters(d):
    """The counter CSV has one row per (dispatch, counter) and only the flat grid size."""
    ds = {}
    for r in csv.DictReader(open(_find(d, "counter_collection.csv"))):
        i = int(r["Dispatch_Id"])
        if i not in ds:
            wgs = int(r["Grid_Size"]) // max(int(r["Workgroup_Size"]), 1)
            ds[i] = Dispatch(_short(r["Kernel_Name"]), None, None, wgs, None)
        ds[i].counters[r["Counter_Name"]] = ds[i].counters.get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
    return _chain(ds)


def pick(ds, sig):
    """Durations of the dispatches that match a signature (kernel, grid, kernel launched before)."""
    _, pat, gx, gy, prev = sig
    return [d.us for d in ds if d.gx == gx and d.gy == gy and re.search(pat, d.name)
            and (prev is None or re.search(prev, d.prev))]


def pick_counter(ds, sig, counter):
    _, pat, gx, gy, prev = sig
    return [d.counters[counter] for d in ds if d.wgs == gx * gy and counter in d.counters and re.search(pat, d.name)
            and (prev is None or re.search(prev, d.prev))]


def copy_factor(ds, counter):
    """KiB the counter reports per KiB moved, from the three 256 MiB device-to-device reference
    copies of --calib-copy (the largest dispatches of the runtime's copy kernel)."""
    big = sorted(d.counters.get(counter, 0.0) for d in ds if "rocclr_copyBuffer" in d.name)[-3:]
    if not big or max(big) <= 0:
        return None
    return (sum(big) / len(big)) / 262144.0


def write_kernel_stats(csv_path, out_dir, cmd):
    """rocprofv3's own per-kernel statistics (--stats) of the traced bench.py run as a short table:
    one row per kernel name, over every workload that launches it."""
    rows = list(csv.DictReader(open(csv_path)))
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    lines = ["# rocprofv3 --kernel-trace --stats: per-kernel statistics of one bench.py run", "",
             "Command (from the repository root on the MI355X box, after `cd /tmp && export TMPDIR=/tmp`):", "",
             "    " + cmd, "",
             "Rows are rocprofv3's `kernel_stats` (one per kernel name, all workloads of the run together; the",
             "per-workload tables in this folder split them by workgroup count). The 30 largest by total time.", "",
             "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---:|---:|---:|---:|---:|"]
    for r in rows[:30]:
        lines.append(f"| `{_short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | "
                     f"{float(r['MinNs']) / 1e3:.1f} | {float(r['MaxNs']) / 1e3:.1f} | {float(r['Percentage']):.2f} |")
    open(os.path.join(out_dir, "kernel_stats_bench.md"), "w").write("\n".join(lines) + "\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--kt", required=True)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--pmc")
    ap.add_argument("--out", required=True)
    ap.add_argument("--note", default="", help="one line appended to every file (the bench line of the traced run)")
    a = ap.parse_args()
    os.makedirs(a.out, exist_ok=True)
    kt = load_trace(a.kt)
    fe = load_counters(a.fetch) if a.fetch else None
    wr = load_counters(a.write) if a.write else None
    pm = load_counters(a.pmc) if a.pmc else None
    ff_ = copy_factor(fe, "FETCH_SIZE") if fe else None
    fw_ = copy_factor(wr, "WRITE_SIZE") if wr else None
    traffic = {}
    cmds = ["rocprofv3 --kernel-trace --stats --output-format csv -d <out> -o kt -- python3 <repo>/bench.py --steps 10 --warmup 3 --no-cpu"]
    if fe:
        cmds.append("rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -o fetch -- python3 <repo>/bench.py --steps 3 --warmup 1 "
                    "--preheat-ms 0 --no-cpu --calib-copy")
    if wr:
        cmds.append("rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out> -o write -- python3 <repo>/bench.py --steps 3 --warmup 1 "
                    "--preheat-ms 0 --no-cpu --calib-copy")
    if pm:
        cmds.append("rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_WAIT_INST_LDS "
                    "SQ_ACTIVE_INST_ANY --output-format csv -d <out> -o pmc -- python3 <repo>/bench.py --steps 3 --warmup 1 "
                    "--preheat-ms 0 --no-cpu")
    for wl_name, sig in SIGNATURES.items():
        lines = [f"# rocprofv3 summary: {wl_name}", "",
                 "Commands (each its own run, from the repository root on the MI355X box, after `cd /tmp && export TMPDIR=/tmp`):", ""]
        lines += ["    " + c for c in cmds]
        lines += ["", f"Summary written by `python -m paper_2401_04044_amd.profile_summary`.", ""]
        head = "| launch | kernel | workgroups | calls | avg us | min us |"
        sep = "|---|---|---:|---:|---:|---:|"
        if fe and wr:
            head += " read MB | written MB |"
            sep += "---:|---:|"
        if pm:
            head += " MFMA busy % | LDS bank conflict cycles | LDS active % |"
            sep += "---:|---:|---:|"
        lines += [head, sep]
        tot_us = tot_r = tot_w = 0.0
        complete = True
        for one in sig:
            one = tuple(one) + (None,) * (5 - len(one))
            label, pat, gx, gy, _ = one
            v = pick(kt, one)
            if not v:
                lines.append(f"| {label} | `{pat}` | {gx}{' x ' + str(gy) if gy > 1 else ''} | 0 | - | - |")
                complete = False
                continue
            avg = sum(v) / len(v)
            tot_us += avg
            row = f"| {label} | `{pat.replace(G, 'gemm_bf16_dl_kernel<')}` | {gx}{' x ' + str(gy) if gy > 1 else ''} | {len(v)} | {avg:.1f} | {min(v):.1f} |"
            if fe and wr:
                f_ = pick_counter(fe, one, "FETCH_SIZE")
                w_ = pick_counter(wr, one, "WRITE_SIZE")
                if f_ and w_ and ff_ and fw_:
                    rmb = sum(f_) / len(f_) * 1024 / ff_ / 1e6
                    wmb = sum(w_) / len(w_) * 1024 / fw_ / 1e6
                    tot_r += rmb
                    tot_w += wmb
                    row += f" {rmb:.1f} | {wmb:.1f} |"
                else:
                    row += " - | - |"
            if pm:
                busy = pick_counter(pm, one, "SQ_BUSY_CU_CYCLES")
                mf = pick_counter(pm, one, "SQ_VALU_MFMA_BUSY_CYCLES")
                bc = pick_counter(pm, one, "SQ_LDS_BANK_CONFLICT")
                la = pick_counter(pm, one, "SQ_LDS_IDX_ACTIVE")
                if busy and mf and sum(busy) > 0:
                    # MFMA busy cycles are summed over the four SIMDs of a CU
                    row += f" {100.0 * sum(mf) / (4.0 * sum(busy)):.1f} | {sum(bc) / max(len(bc), 1):.0f} | {100.0 * sum(la) / (4.0 * sum(busy)):.1f} |"
                else:
                    row += " - | - | - |"
            lines.append(row)
        if wl_name != "ceilings":
            tail = f"| **sum of the launches of one call** | | | | **{tot_us:.1f}** | |"
            if fe and wr:
                tail += f" **{tot_r:.1f}** | **{tot_w:.1f}** |"
            if pm:
                tail += " | | |"
            lines.append(tail)
        if fe and wr and ff_ and fw_:
            lines += ["", f"Counter scaling from the 256 MiB reference copy (`--calib-copy`): FETCH_SIZE reports {ff_:.3f} KiB per KiB read, "
                          f"WRITE_SIZE {fw_:.3f} KiB per KiB written; the MB columns are divided by these."]
            if complete and wl_name in TRAFFIC_KEYS:
                keys = TRAFFIC_KEYS[wl_name]
                for k in ([keys] if isinstance(keys, str) else keys):
                    traffic[k] = (tot_r + tot_w) * 1e6
        if pm:
            lines += ["", "MFMA busy % = SQ_VALU_MFMA_BUSY_CYCLES / (4 x SQ_BUSY_CU_CYCLES) (the pure-MFMA probe reads 100 %); "
                          "LDS active % likewise from SQ_LDS_IDX_ACTIVE."]
        if a.note:
            lines += ["", a.note]
        open(os.path.join(a.out, wl_name + ".md"), "w").write("\n".join(lines) + "\n")
    stats = glob.glob(os.path.join(a.kt, "*kernel_stats.csv"))
    if stats:
        write_kernel_stats(stats[0], a.out, cmds[0])
    if traffic:
        json.dump(traffic, open(os.path.join(a.out, "hbm_traffic.json"), "w"), indent=1, sort_keys=True)
    print("wrote", ", ".join(sorted(SIGNATURES)), "and", "hbm_traffic.json" if traffic else "no traffic file")


if __name__ == "__main__":
    main()
