"""Turns rocprofv3 output of bench.py runs into the short summaries under profiles/ and profiles/traffic.json.

    python -m paper_2504_12397_amd.profile_summary --in <directory with the rocprofv3 output> --out profiles

Expects under --in, per workload w in {c2, c3, c4, c5, r3p, r3pp} (any subset; r3p and r3pp are bench.py's r3p workload with
--variant shared and --variant private):
    kt_<w>/<w>_kernel_stats.csv, kt_<w>.json          rocprofv3 --kernel-trace --stats, and bench.py's JSON line
    pmc_FETCH_<w>/, pmc_WRITE_<w>/                    --pmc FETCH_SIZE / WRITE_SIZE  (<w>_counter_collection.csv)
    pmc_A_<w>/, pmc_B_<w>/                            the two sets of SQ counters listed in COUNTER_SETS
and pmc_FETCH_copy/, pmc_WRITE_copy/ (bench.py --workload copy) to calibrate the two HBM counters.
The commands are printed into every summary.  bench.py reads traffic.json for roofline.traffic.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import re

N_CU, N_XCD = 256, 8
COUNTER_SETS = {
    "A": "SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_VALU_MFMA_COEXEC_CYCLES SQ_INSTS_VALU_MFMA_MOPS_F16 "
         "SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT GRBM_GUI_ACTIVE",
    "B": "SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_ACTIVE_INST_VMEM SQ_LDS_IDX_ACTIVE SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS "
         "SQ_INSTS_VALU SQ_INSTS_MFMA GRBM_GUI_ACTIVE",
}
TITLES = {
    "c2": ("c2_prefill_layer", "c2: one 8B-class layer, 4096 cached base tokens + 256 adapted suffix tokens, rank 32", ""),
    "c3": ("c3_mixed_batch", "c3: mixed batch, 16 sequences, prefix 512-8192, suffix 32-512, 4 rank-32 adapters, 3 base-only", ""),
    "c4": ("c4_decode_step", "c4: decode step, 64 sequences x 16448 cached tokens, one new token each", ""),
    "c5": ("c5_stack_first_token", "c5: 32-layer 8B-class stack, 32768 cached base tokens + 128 adapted suffix tokens, rank 64",
           " --only --no-full-lora"),
    "r3p": ("r3p_shared_context_prefill", "r3p: prefill of 32 invocation sequences of 16 tokens, 4 contexts of 16384 cached base "
            "tokens x 8 adapter calls, each context's rows stored once and walked once per run of sequences", " --variant shared"),
    "r3pp": ("r3p_private_copies_prefill", "r3p with private copies: the same 32 invocation sequences, every sequence holding "
             "(and walking) its own copy of the 16384 context rows", " --variant private"),
}
BENCH_WORKLOAD = {"r3pp": "r3p"}         # summary key -> bench.py --workload, where they differ
# kernel symbol -> the kernel family bench.py reports (only where one symbol is one family in that workload)
FAMILY = [("attn_prefill_mfma_kernel", "attn_prefill"), ("attn_decode_mfma_kernel", "attn_decode"),
          ("prep_rows_mfma_kernel", "prep_rows"), ("rope_append_kernel", "rope_append"), ("attn_merge", "attn_merge")]


def short(name: str) -> str:
    n = name.replace("void ", "")
    m = re.match(r"_ZN5alora(\d+)", n)
    if m:
        k = int(m.group(1))
        n = "alora::" + n[len(m.group(0)):len(m.group(0)) + k]
    n = re.sub(r"\(.*", "", n)
    return n[:72]


def family_of(workload: str, kernel: str):
    for pat, fam in FAMILY:
        if pat in kernel:
            return fam
    if "gemm_mfma_kernel" in kernel:
        epi = re.search(r"gemm_mfma_kernel<\d+, \d+, \d+, \d+, (\d),", kernel)
        epi = epi.group(1) if epi else ""
        if workload == "c3":
            return "qkv_gemm"
        if workload in ("c2", "c4") and epi == "0":       # (c2 also runs a 4096-row base prefill at set-up: epilogue 3)
            return "qkv_gemm"
        if workload == "c5" and epi == "2":
            return "gate_up"
    return None


def kernel_stats(path):
    rows = []
    for r in csv.DictReader(open(path)):
        if "alora" in r["Name"]:
            rows.append((short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]), float(r["Percentage"])))
    return rows


def counters(path, keep_all=False):
    """{kernel: {counter: mean over the later half of its dispatches}}"""
    d = collections.defaultdict(lambda: collections.defaultdict(list))
    if not os.path.exists(path):
        return {}
    for r in csv.DictReader(open(path)):
        n = r["Kernel_Name"]
        if "alora" in n or keep_all:
            d[short(n)][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: sum(v[len(v) // 2:]) / len(v[len(v) // 2:]) for c, v in cs.items()} for k, cs in d.items()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--in", dest="src", default="gpurun_out/prof")
    ap.add_argument("--out", default="profiles")
    args = ap.parse_args()
    src = args.src

    def cal(counter):
        d = counters(f"{src}/pmc_{counter}_copy/copy_counter_collection.csv", keep_all=True)
        vals = [cs.get(f"{counter}_SIZE", 0.0) for cs in d.values()]
        return max(vals) if vals else None

    fcal, wcal = cal("FETCH"), cal("WRITE")
    fs = 1048576.0 / fcal if fcal else None
    ws = 1048576.0 / wcal if wcal else None
    traffic = {}
    for w, (fname, title, extra) in TITLES.items():
        kt = f"{src}/kt_{w}/{w}_kernel_stats.csv"
        if not os.path.exists(kt):
            continue
        ks = kernel_stats(kt)
        j = json.loads(open(f"{src}/kt_{w}.json").read().strip().splitlines()[-1])
        fetch = counters(f"{src}/pmc_FETCH_{w}/{w}_counter_collection.csv")
        write = counters(f"{src}/pmc_WRITE_{w}/{w}_counter_collection.csv")
        ca = counters(f"{src}/pmc_A_{w}/{w}_counter_collection.csv")
        cb = counters(f"{src}/pmc_B_{w}/{w}_counter_collection.csv")
        pmc_extra = extra + (" --layers 4" if w == "c5" else "")
        bw = BENCH_WORKLOAD.get(w, w)
        out = [f"# rocprofv3 summary, workload {title}", "",
               "Commands (from /tmp with TMPDIR=/tmp on one MI355X; paths relative to the repository root; every --pmc pass is a run of its own):", "",
               f"    rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof/kt_{w} -o {w} -- python3 bench.py --workload {bw} --no-cpu-baseline{extra}",
               f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/prof/pmc_FETCH_{w} -o {w} -- python3 bench.py --workload {bw} --no-cpu-baseline --steps 3 --warmup 1{pmc_extra}",
               "    (the same with WRITE_SIZE, and with the two SQ counter sets below)",
               f"    set A: {COUNTER_SETS['A']}",
               f"    set B: {COUNTER_SETS['B']}",
               "    python3 -m paper_2504_12397_amd.profile_summary --in gpurun_out/prof --out profiles", ""]
        if fs and ws:
            out += [f"HBM counter calibration on `python3 bench.py --workload copy` (1 GiB copied = 1048576 KiB read and written per "
                    f"dispatch): FETCH_SIZE reads {fcal:.0f}, WRITE_SIZE reads {wcal:.0f}, so they are scaled by {fs:.2f} and {ws:.2f}.", ""]
        rl = j["roofline"]
        out += [f"bench.py under the kernel-trace run: {j['ms_per_step']:.4f} ms per step, {j['value']:.0f} tok/s; dominant kernel "
                f"`{rl['kernel']}` {rl['achieved']:.1f} {rl['unit']} = {100 * rl['frac']:.1f} % of the published peak (HIP events inside bench.py).", "",
                "| kernel | calls | avg µs (rocprofv3) | bench.py events µs | % of trace | HBM read MB | HBM written MB | clock GHz | MFMA busy % | MFMA+VALU co-issue % | VALU active % | LDS active % | LDS bank conflict % | waiting % of wave cycles |",
                "|---|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
        # one kernel symbol per family: where set-up code ran another variant of a kernel, the one with most calls counts
        most = {}
        for n, calls, avg, pct in ks:
            fam = family_of(w, n)
            if fam and calls > most.get(fam, ("", -1))[1]:
                most[fam] = (n, calls)
        for n, calls, avg, pct in ks:
            fam = family_of(w, n)
            if fam and most[fam][0] != n:
                fam = None
            ev = f"{fam} = {j['kernels'][fam]['avg_ms'] * 1e3:.1f}" if fam and fam in j.get("kernels", {}) else ""
            fb = fs * fetch.get(n, {}).get("FETCH_SIZE", 0.0) * 1024 if fs and n in fetch else None
            wb = ws * write.get(n, {}).get("WRITE_SIZE", 0.0) * 1024 if ws and n in write else None
            a, b = ca.get(n, {}), cb.get(n, {})
            cols = [""] * 7
            gui = a.get("GRBM_GUI_ACTIVE") or b.get("GRBM_GUI_ACTIVE")
            if gui:
                cyc = gui / N_XCD                      # the counter is summed over the XCDs
                if avg >= 50e3:
                    cols[0] = f"{cyc / avg:.2f}"
                else:
                    cyc = avg * 2.4                    # short kernel: the counter also covers its launch; nominal clock instead
                if "SQ_VALU_MFMA_BUSY_CYCLES" in a:
                    cols[1] = f"{100 * a['SQ_VALU_MFMA_BUSY_CYCLES'] / (cyc * N_CU * 4):.1f}"
                    cols[2] = f"{100 * a.get('SQ_VALU_MFMA_COEXEC_CYCLES', 0) / (cyc * N_CU * 4):.1f}"
                if "SQ_ACTIVE_INST_VALU" in b:
                    cols[3] = f"{100 * 4 * b['SQ_ACTIVE_INST_VALU'] / (cyc * N_CU * 4):.1f}"
                if "SQ_LDS_IDX_ACTIVE" in b:
                    cols[4] = f"{100 * b['SQ_LDS_IDX_ACTIVE'] / (cyc * N_CU):.1f}"
                    if "SQ_LDS_BANK_CONFLICT" in a:
                        cols[5] = f"{100 * a['SQ_LDS_BANK_CONFLICT'] / max(b['SQ_LDS_IDX_ACTIVE'], 1):.1f}"
                if "SQ_WAIT_INST_ANY" in b and "SQ_WAVE_CYCLES" in a:
                    cols[6] = f"{100 * b['SQ_WAIT_INST_ANY'] / max(a['SQ_WAVE_CYCLES'], 1):.0f}"
            out.append(f"| `{n}` | {calls} | {avg / 1e3:.1f} | {ev} | {pct:.1f} | "
                       f"{'' if fb is None else f'{fb / 1e6:.1f}'} | {'' if wb is None else f'{wb / 1e6:.1f}'} | " + " | ".join(cols) + " |")
            if fam and fb is not None and wb is not None:
                traffic[f"{w}/{fam}"] = {"kernel": n, "fetch_bytes": round(fb), "write_bytes": round(wb),
                                         "fetch_scale": round(fs, 3), "write_scale": round(ws, 3)}
        out += ["", "Columns: clock = GRBM_GUI_ACTIVE / 8 XCDs / duration; MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (cycles x 256 CUs x 4 SIMDs); "
                "(kernels under 50 µs: cycles = duration x 2.4 GHz, the counter also covers their launch); co-issue = SQ_VALU_MFMA_COEXEC_CYCLES over the same; VALU active = 4 x SQ_ACTIVE_INST_VALU over the same; LDS active = "
                "SQ_LDS_IDX_ACTIVE / (cycles x 256 CUs); bank conflict = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE; waiting = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES."]
        if w == "c5":
            out += ["The counter runs use 4 layers (`--layers 4`); per-launch figures do not depend on the layer count."]
        open(os.path.join(args.out, fname + ".md"), "w").write("\n".join(out) + "\n")
        print("wrote", fname)
    if traffic:
        json.dump(traffic, open(os.path.join(args.out, "traffic.json"), "w"), indent=1, sort_keys=True)
        print("wrote traffic.json with", len(traffic), "entries")


if __name__ == "__main__":
    main()
