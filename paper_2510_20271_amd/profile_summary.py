"""Turns rocprofv3 output into the short summaries under profiles/ and into profiles/counters.json
(the counter-based figures bench.py reports: HBM traffic per launch, VALU / LDS instruction counts).

    python -m paper_2510_20271_amd.profile_summary --commands [OUT]   print the rocprofv3 commands (one run per line)
    python -m paper_2510_20271_amd.profile_summary OUT                summarise the CSVs those runs left under OUT

Every run profiles `python3 bench.py --only <workload>`.  rocprofv3 does not split counters over
passes, so each counter set is a run of its own: a kernel trace (durations), the SQ / GRBM
instruction counters, FETCH_SIZE and WRITE_SIZE; two more runs on a plain 1 GiB device copy
(`--only calib`) calibrate the two size counters.
"""
from __future__ import annotations

import collections
import csv
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SQ = ("SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_WAVES SQ_ACTIVE_INST_VALU SQ_BUSY_CYCLES SQ_LDS_BANK_CONFLICT "
      "SQ_ACTIVE_INST_LDS GRBM_GUI_ACTIVE")

# workload -> (title, file, [(counters.json key, kernel-name fragment, vertices per launch or None, lanes of a wave row)])
WORKLOADS = {
    "c2": ("hard ECC, workload C2 (16 x 4096^2 float32, 1024 bins, range found on the device)", "hard_c2.md",
           [("c2", "sweep2d_list_kernel", 16 * 4096 * 4096, 248)]),
    "c2r": ("hard ECC, workload C2 with the range supplied (histogram-mode sweep)", "hard_c2_range.md",
            [("c2r", "sweep2d_kernel", 16 * 4096 * 4096, 248)]),
    "c4": ("hard ECC, workload C4 (512^3 float32, 1024 bins, range found on the device)", "hard_c4.md",
           [("c4", "sweep3d_list_kernel", 512 ** 3, 62)]),
    "c4r": ("hard ECC, workload C4 with the range supplied (histogram-mode sweep)", "hard_c4_range.md",
            [("c4r", "sweep3d_kernel", 512 ** 3, 62)]),
    "c3": ("hard ECC, workload C3 (256^3 uint16 i.i.d., 4096 levels)", "hard_c3.md",
           [("c3", "sweep3d_kernel<unsigned short", 256 ** 3, 62)]),
    "c1": ("hard ECC, workload C1 (256^2 uint8 i.i.d., 256 levels)", "hard_c1.md",
           [("c1", "sweep_generic_kernel", 256 * 256, 64)]),
    "c5": ("soft ECC forward + backward, workload C5 (32 x 512^2 float32, T = 128)", "soft_c5.md",
           [("c5_fwd", "soft2d_fwd_kernel", 32 * 512 * 512, 248), ("c5_bwd", "soft2d_bwd_kernel", 32 * 512 * 512, 248),
            ("c5_fwd_save", "soft2d_fwd_save_kernel", 32 * 512 * 512, 248),
            ("c5_bwd_saved", "soft2d_bwd_saved_kernel", 32 * 512 * 512, 248)]),
    # kernel trace only: the launches behind every row of the size table
    "sizes": ("hard ECC, the grid sizes of the paper's Tables 1-2 (one float32 field per size, 1024 bins, range found on "
              "the device): two launches up to 256^2, three up to 8192^2 / 256^3, five beyond", "hard_sizes.md", []),
}


def commands(out):
    rows = []
    for wl in list(WORKLOADS) + ["calib"]:
        base = f"-- python3 bench.py --only {wl}"
        if wl != "calib":
            rows.append(f"rocprofv3 --kernel-trace --stats --output-format csv -d {out}/{wl}_trace -o {wl} {base} --steps 20")
            if not WORKLOADS[wl][2]:
                continue
            rows.append(f"rocprofv3 --pmc {SQ} --output-format csv -d {out}/{wl}_sq -o {wl} {base} --steps 3 --warmup 1")
        rows.append(f"rocprofv3 --pmc FETCH_SIZE --output-format csv -d {out}/{wl}_fetch -o {wl} {base} --steps 3 --warmup 1")
        rows.append(f"rocprofv3 --pmc WRITE_SIZE --output-format csv -d {out}/{wl}_write -o {wl} {base} --steps 3 --warmup 1")
    return rows


def short(name):
    return name.split("(")[0].replace("void ", "").strip()


def read_pmc(path):
    d = collections.defaultdict(list)
    if not os.path.exists(path):
        return {}
    for r in csv.DictReader(open(path)):
        d[(short(r["Kernel_Name"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in d.items()}


def read_stats(path):
    rows = []
    if not os.path.exists(path):
        return rows
    for r in csv.DictReader(open(path)):
        n = short(r["Name"])
        if n.startswith("at::") or "rocclr" in n or "elementwise" in n:
            continue
        rows.append((n, int(r["Calls"]), float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3,
                     float(r["Percentage"])))
    return rows


def is_kernel(name, frag):
    """frag: a kernel's base name, optionally with the start of its template list."""
    base = name.split("<")[0].split("::")[-1]
    return base == frag.split("<")[0] and ("<" not in frag or frag in name)


def pick(table, frag, counter):
    for (k, c), v in table.items():
        if c == counter and is_kernel(k, frag):
            return v
    return None


def main():
    args = sys.argv[1:]
    if args and args[0] == "--commands":
        print("\n".join(commands(args[1] if len(args) > 1 else "gpurun_out/prof")))
        return
    out = args[0]
    rel = os.path.relpath(out, ROOT) if os.path.isabs(out) else out
    cal_f = read_pmc(f"{out}/calib_fetch/calib_counter_collection.csv")
    cal_w = read_pmc(f"{out}/calib_write/calib_counter_collection.csv")
    kf = [v for (k, c), v in cal_f.items() if "copyBuffer" in k]
    kw = [v for (k, c), v in cal_w.items() if "copyBuffer" in k]
    sf = 1048576.0 / kf[0] if kf else 2.0
    sw = 1048576.0 / kw[0] if kw else 1.0
    result = {"calibration": {"fetch_scale": round(sf, 4), "write_scale": round(sw, 4),
                              "note": "a plain 1 GiB device copy (__amd_rocclr_copyBuffer) reads FETCH_SIZE = %s KiB and "
                                      "WRITE_SIZE = %s KiB for 1048576 KiB moved each way" % (kf[0] if kf else "n/a",
                                                                                            kw[0] if kw else "n/a")},
              "kernels": {}}
    cmds = commands(rel)
    for wl, (title, fname, kernels) in WORKLOADS.items():
        stats = read_stats(f"{out}/{wl}_trace/{wl}_kernel_stats.csv")
        sq = read_pmc(f"{out}/{wl}_sq/{wl}_counter_collection.csv")
        fe = read_pmc(f"{out}/{wl}_fetch/{wl}_counter_collection.csv")
        wr = read_pmc(f"{out}/{wl}_write/{wl}_counter_collection.csv")
        if not (stats or sq or fe):
            continue
        s = f"# rocprofv3 summary: {title}\n\nCommands (each counter set is a run of its own; run from the repository root):\n\n"
        for c in cmds:
            if f"--only {wl} " in c:
                s += f"- `{c}`\n"
        if kernels:
            s += f"- calibration of the size counters: the FETCH_SIZE / WRITE_SIZE commands with `--only calib` (a plain 1 GiB "
            s += f"device copy): scale factors {sf:.3f} (fetch) and {sw:.3f} (write).\n"
        s += "\n"
        if stats:
            s += "Kernel durations (kernel trace):\n\n| kernel | calls | avg us | min us | max us | % |\n|---|---|---|---|---|---|\n"
            for n, c, a, mi, ma, p in stats:
                s += f"| `{n}` | {c} | {a:.1f} | {mi:.1f} | {ma:.1f} | {p:.1f} |\n"
            s += "\n"
        for key, frag, nvert, lanes in kernels:
            entry = {"kernel": frag}
            avg = [a for n, c, a, mi, ma, p in stats if is_kernel(n, frag)]
            if avg:
                entry["avg_us"] = round(avg[0], 2)
            f = pick(fe, frag, "FETCH_SIZE")
            w = pick(wr, frag, "WRITE_SIZE")
            if f is not None and w is not None:
                entry["fetch_bytes"] = round(f * sf * 1024)
                entry["write_bytes"] = round(w * sw * 1024)
            names = SQ.split()
            vals = {c: pick(sq, frag, c) for c in names}
            for c, v in vals.items():
                if v is not None:
                    entry[c] = round(v)
            s += f"## `{frag}`\n\n| counter (per launch, summed over the chip) | value |\n|---|---|\n"
            for c in names:
                if vals[c] is not None:
                    s += f"| {c} | {vals[c]:.0f} |\n"
            if "fetch_bytes" in entry:
                s += f"| FETCH_SIZE x {sf:.3f} (bytes) | {entry['fetch_bytes']} |\n| WRITE_SIZE x {sw:.3f} (bytes) | {entry['write_bytes']} |\n"
            s += "\n"
            if vals.get("SQ_INSTS_VALU") and vals.get("GRBM_GUI_ACTIVE"):
                cyc = vals["GRBM_GUI_ACTIVE"] / 8  # the counter adds up the eight XCDs
                util = vals["SQ_INSTS_VALU"] * 4 / (1024 * cyc)
                entry["valu_issue_utilisation"] = round(util, 3)
                s += (f"GRBM_GUI_ACTIVE counts every XCD: {cyc:.0f} cycles per XCD for the launch (with the counters "
                      f"running; the kernel trace above has the undisturbed duration).  ")
                if nvert:
                    per = vals["SQ_INSTS_VALU"] / (nvert / lanes)
                    entry["valu_per_wave_row"] = round(per, 1)
                    s += f"VALU instructions per {lanes}-vertex wave row: {per:.1f}.  "
                s += (f"VALU issue utilisation, taking 4 cycles per wave instruction on each of the 1024 SIMDs: {util:.2f}.")
                if vals.get("SQ_INSTS_LDS"):
                    s += (f"  LDS: {vals['SQ_INSTS_LDS']:.0f} instructions, {vals.get('SQ_ACTIVE_INST_LDS') or 0:.0f} busy cycles, "
                          f"{vals.get('SQ_LDS_BANK_CONFLICT') or 0:.0f} of them bank conflicts (summed over 256 CUs).")
                s += "\n\n"
            if "fetch_bytes" in entry and nvert:
                s += (f"HBM traffic per launch: {(entry['fetch_bytes'] + entry['write_bytes']) / 1e6:.1f} MB "
                      f"({entry['fetch_bytes'] / 1e6:.1f} read + {entry['write_bytes'] / 1e6:.1f} written).\n\n")
            result["kernels"][key] = entry
        open(os.path.join(ROOT, "profiles", fname), "w").write(s)
        print("wrote profiles/" + fname)
    json.dump(result, open(os.path.join(ROOT, "profiles", "counters.json"), "w"), indent=1)
    print("wrote profiles/counters.json")


if __name__ == "__main__":
    main()
