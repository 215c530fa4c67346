#!/usr/bin/env python3
"""Turns the per-dispatch CSV files of `rocprofv3 --pmc ... -- python3 bench.py --workload W ...` runs into the short
text summaries under profiles/ and into profiles/counters.json, which bench.py reads for `roofline.traffic` and
`roofline.mfma_util`. Usage (one rocprofv3 run per counter group, each writing <dir>/<W>_<group>_counter_collection.csv):

    cd /tmp && export TMPDIR=/tmp && cd <repo>
    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_VALU SQ_INSTS_SALU \
              SQ_WAVE_CYCLES SQ_LDS_BANK_CONFLICT GRBM_GUI_ACTIVE \
              -d <dir> -o W_sq --output-format csv -- python3 bench.py --workload W --steps 2 --warmup 1 --no-cpu-baseline
    rocprofv3 --pmc FETCH_SIZE -d <dir> -o W_fetch --output-format csv -- python3 bench.py --workload W --steps 2 --warmup 1 --no-cpu-baseline
    rocprofv3 --pmc WRITE_SIZE -d <dir> -o W_write --output-format csv -- python3 bench.py --workload W --steps 2 --warmup 1 --no-cpu-baseline
    python3 bench_counters.py <dir> W [W ...]

Calibration comes from the same runs: bench.py starts with one plain 1 GiB device copy (what FETCH_SIZE / WRITE_SIZE
read for a known number of bytes) and with the library's register-only MFMA loop (what the MFMA counters read for a
kernel that keeps every matrix core busy and whose flop count is known)."""
import collections
import csv
import json
import os
import sys

from bench import kernel_sources_digest

ROOT = os.path.dirname(os.path.abspath(__file__))
csv.field_size_limit(1 << 30)

# stage name of bench.py -> substring of the kernel that dominates it
DOMINANT = {"gate_up_gemm": "EpiSiluMul", "attention_topk": "k_attn_decode<", "attention_select": "k_attn_select<",
            "prune_quant": "k_prune_fq_wave", "down_gemm": "EpiResidOut", "lm_head_gemm": "EpiNllCols"}
TITLES = {"c2": "C2 (one Llama-3.2-1B-shaped layer, 32 x 1024 tokens)", "c3": "C3 (16-layer stack + LM head, 16 x 2048 tokens)",
          "c4": "C4 (decode step, 64 x 8192-token caches, 16 layers + LM head)", "c5": "C5 (one Llama-3.1-8B-shaped layer, 8 x 4096 tokens)",
          "c5d": "C5-decode (one 8B-shaped layer, 32 x 8192-token caches)", "c2p": "C2, the paper's own configuration",
          "c4p": "C4, the paper's own configuration with page metadata"}


def short(name):
    name = name.replace("unsigned short", "bf16").replace("void ", "")
    return (name.split("(")[0] if name.startswith("at::") else name)[:96]


def load(path):
    """{kernel: {counter: [value per dispatch]}}"""
    d = collections.defaultdict(lambda: collections.defaultdict(list))
    if not os.path.exists(path):
        return d
    per = collections.defaultdict(dict)
    for r in csv.DictReader(open(path)):
        per[(r["Dispatch_Id"], short(r["Kernel_Name"]))][r["Counter_Name"]] = float(r["Counter_Value"])
    for (_, k), c in per.items():
        for n, v in c.items():
            d[k][n].append(v)
    return d


def avg(v):
    return sum(v) / len(v) if v else 0.0


def main():
    src, workloads = sys.argv[1], sys.argv[2:]
    path = os.path.join(ROOT, "profiles", "counters.json")
    try:
        out = json.load(open(path))
    except (OSError, ValueError):
        out = {}
    digest = kernel_sources_digest()
    if out.get("kernel_sources_digest") != digest:
        out = {"kernel_sources_digest": digest}
    for wl in workloads:
        sq, fe, wr = (load(os.path.join(src, f"{wl}_{g}_counter_collection.csv")) for g in ("sq", "fetch", "write"))
        cmd = "python3 bench.py --workload %s --steps 2 --warmup 1 --no-cpu-baseline" % wl
        lines = ["rocprofv3 --pmc summary per kernel launch (MI355X, gfx950), workload %s" % TITLES.get(wl, wl),
                 "commands (one run per counter group; cd /tmp && export TMPDIR=/tmp && cd <repo> first):",
                 "  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_VALU SQ_INSTS_SALU "
                 "SQ_WAVE_CYCLES SQ_LDS_BANK_CONFLICT GRBM_GUI_ACTIVE -d <dir> -o %s_sq --output-format csv -- %s" % (wl, cmd),
                 "  rocprofv3 --pmc FETCH_SIZE -d <dir> -o %s_fetch --output-format csv -- %s" % (wl, cmd),
                 "  rocprofv3 --pmc WRITE_SIZE -d <dir> -o %s_write --output-format csv -- %s" % (wl, cmd),
                 "  python3 bench_counters.py <dir> %s" % wl]
        # calibration kernels
        copy = next((k for k in fe if "copyBuffer" in k), None)
        sf = 1048576.0 / max(fe[copy]["FETCH_SIZE"]) if copy else None
        cw = next((k for k in wr if "copyBuffer" in k), None)
        sw = 1048576.0 / max(wr[cw]["WRITE_SIZE"]) if cw else None
        if sf and sw:
            lines.append("calibration, HBM: the 1 GiB device copy reads FETCH_SIZE = %.1f and WRITE_SIZE = %.1f for 1048576 KiB each "
                         "way: scale factors %.4f (fetch) and %.4f (write)" % (1048576.0 / sf, 1048576.0 / sw, sf, sw))
        pk = next((k for k in sq if "k_peak_mfma" in k), None)
        busy_per_cycle = mops_flops = None
        if pk:
            c = sq[pk]
            # the timed launches of the loop (4096 rounds) dominate; the 64-round warm-up launch is the smallest
            i = max(range(len(c["GRBM_GUI_ACTIVE"])), key=lambda j: c["GRBM_GUI_ACTIVE"][j])
            busy_per_cycle = c["SQ_VALU_MFMA_BUSY_CYCLES"][i] / c["GRBM_GUI_ACTIVE"][i]
            waves = c["SQ_WAVES"][i] if "SQ_WAVES" in c else None
            lines.append("calibration, MFMA: the register-only MFMA loop (every matrix core busy) reads SQ_VALU_MFMA_BUSY_CYCLES / "
                         "GRBM_GUI_ACTIVE = %.2f; a kernel's mfma_util is its own ratio divided by this one" % busy_per_cycle)
            del waves
        lines += ["", "columns: launches | avg GRBM_GUI_ACTIVE (cycles) | mfma_util | MFMA_MOPS_BF16 | INSTS_VALU | INSTS_SALU | "
                  "WAVE_CYCLES | LDS_BANK_CONFLICT | fetch MiB | write MiB | kernel", ""]
        names = [k for k in set(sq) | set(fe) | set(wr) if k.startswith("sol::")]
        names.sort(key=lambda k: -avg(sq[k]["GRBM_GUI_ACTIVE"]) * len(sq[k]["GRBM_GUI_ACTIVE"]))
        rec = {}
        for k in names:
            c = sq[k]
            act = avg(c["GRBM_GUI_ACTIVE"])
            util = (avg(c["SQ_VALU_MFMA_BUSY_CYCLES"]) / act / busy_per_cycle) if (act and busy_per_cycle) else None
            fm = avg(fe[k]["FETCH_SIZE"]) * sf / 1024 if (sf and k in fe) else None
            wm = avg(wr[k]["WRITE_SIZE"]) * sw / 1024 if (sw and k in wr) else None
            lines.append("%-5d %12.0f %7s %14.0f %14.0f %14.0f %16.0f %12.0f %10s %10s  %s" % (
                len(c["GRBM_GUI_ACTIVE"]) or len(fe[k]["FETCH_SIZE"]), act, "%.3f" % util if util is not None else "-",
                avg(c["SQ_INSTS_VALU_MFMA_MOPS_BF16"]), avg(c["SQ_INSTS_VALU"]), avg(c["SQ_INSTS_SALU"]), avg(c["SQ_WAVE_CYCLES"]),
                avg(c["SQ_LDS_BANK_CONFLICT"]), "%.1f" % fm if fm is not None else "-",
                "%.1f" % wm if wm is not None else "-", k))
            for stage, match in DOMINANT.items():
                if match in k and stage not in rec:
                    rec[stage] = {"kernel": k, "mfma_util": util,
                                  "traffic": int((fm + wm) * (1 << 20)) if fm is not None and wm is not None else None,
                                  "fetch_bytes": int(fm * (1 << 20)) if fm is not None else None,
                                  "write_bytes": int(wm * (1 << 20)) if wm is not None else None,
                                  "insts_valu": avg(c["SQ_INSTS_VALU"]) or None, "insts_salu": avg(c["SQ_INSTS_SALU"]) or None,
                                  "gui_active_cycles": act or None}
        # MFMA flops the whole step executed (SQ_INSTS_VALU_MFMA_MOPS_BF16 counts units of 512 flops: the gate_up GEMM's
        # 2^32 per launch are its 2 * 32768 * 2048 * 16384 flops), over all kernels of the library; steps run in the
        # profiled process = launches of k_prepare_rows, which every entry point launches once
        n_steps = next((len(sq[k]["GRBM_GUI_ACTIVE"]) for k in names if "k_prepare_rows" in k), 0)
        if n_steps:
            mops = sum(sum(sq[k]["SQ_INSTS_VALU_MFMA_MOPS_BF16"]) for k in names if "k_peak_" not in k)   # not the peak microbenchmarks
            rec["step"] = {"mfma_executed_flops": mops * 512.0 / n_steps, "steps_profiled": n_steps}
            lines += ["", "MFMA flops executed per step, all kernels (MFMA_MOPS_BF16 x 512 / %d steps): %.3f TFLOP" % (
                n_steps, mops * 512.0 / n_steps / 1e12)]
        # the step's traffic by the same counters, all kernels (scaled as above), for the HBM-bound records
        nf = next((len(fe[k]["FETCH_SIZE"]) for k in fe if "k_prepare_rows" in k), 0)
        nw = next((len(wr[k]["WRITE_SIZE"]) for k in wr if "k_prepare_rows" in k), 0)
        if sf and sw and nf and nw:
            fb = sum(sum(fe[k]["FETCH_SIZE"]) for k in fe if k.startswith("sol::") and "k_peak_" not in k) * sf * 1024.0 / nf
            wb = sum(sum(wr[k]["WRITE_SIZE"]) for k in wr if k.startswith("sol::") and "k_peak_" not in k) * sw * 1024.0 / nw
            rec.setdefault("step", {}).update({"fetch_bytes": fb, "write_bytes": wb})
            lines += ["bytes fetched / written per step, all kernels: %.3f / %.3f GB" % (fb / 1e9, wb / 1e9)]
        out[wl] = rec
        txt = os.path.join(ROOT, "profiles", "%s_counters.txt" % wl)
        open(txt, "w").write("\n".join(lines) + "\n")
        print(open(txt).read())
    json.dump(out, open(path, "w"), indent=1)


if __name__ == "__main__":
    main()
