"""Summarise rocprofv3 CSV output of a bench.py run.

    python profile_summary.py stats  <dir>/<prefix>_kernel_stats.csv
    python profile_summary.py pmc    <fetch>_counter_collection.csv <write>_counter_collection.csv
                                                          [kernel name prefix = gemm_bf16 [largest]]

    python profile_summary.py counters <counter_collection.csv> [more .csv ...]
    python profile_summary.py durations <dir>/<prefix>_kernel_trace.csv <kernel name prefix> [<bytes per launch>]
    python profile_summary.py streaming <dir>/<prefix>_kernel_trace.csv <tokens> <d_model> <d_ffn>

`durations` prints a JSON object with the number of launches, the average, median and minimum kernel duration
(End_Timestamp - Start_Timestamp of the kernel trace) of the kernels whose name starts with the prefix, and GB/s
for the given algorithmic bytes per launch.  `streaming` prints a table of the HBM-bound kernels of a stage step
(LayerNorm, column sums, codec, attention row sums) with their algorithmic bytes per launch and GB/s against 8 TB/s.

`counters` prints, per kernel family (GEMM: per instantiation; others: name up to the template arguments), the sum over all launches of every
counter found in the given rocprofv3 --pmc runs of bench.py, and each counter as a fraction of SQ_BUSY_CU_CYCLES
(per-CU busy cycles) resp. of SQ_WAVE_CYCLES where those are present in the same file.

`pmc` expects two runs of `bench.py --copy-calibration` under `rocprofv3 --pmc FETCH_SIZE` and
`--pmc WRITE_SIZE`.  The counters are scaled by what they read for the plain 1 GiB device copies of
that run (each reads 2^30 and writes 2^30 bytes), then averaged over the launches of the kernels whose name starts
with the prefix (with `largest`: only over the launches with the largest grid, i.e. the largest tensor).
"""
from __future__ import annotations

import collections
import csv
import json
import sys

GIB = float(1 << 30)


def _short(name: str) -> str:
    return name.replace("swarm::(anonymous namespace)::", "").replace("void ", "").split("(")[0]


def stats(path: str) -> None:
    rows = list(csv.DictReader(open(path)))
    print("| kernel | calls | avg us | total ms | % |")
    print("|---|---|---|---|---|")
    g_ns, g_calls = 0.0, 0
    for r in rows:
        if float(r["Percentage"]) < 0.05:
            continue
        n = _short(r["Name"])
        print("| `%s` | %s | %.1f | %.2f | %.1f |" % (n, r["Calls"], float(r["AverageNs"]) / 1e3,
                                                    float(r["TotalDurationNs"]) / 1e6, float(r["Percentage"])))
        if n.startswith("gemm_bf16"):
            g_ns += float(r["TotalDurationNs"])
            g_calls += int(r["Calls"])
    if g_calls:
        print("\nAll bf16 GEMM kernels: %d calls, average %.1f us per launch." % (g_calls, g_ns / g_calls / 1e3))


def _per_kernel(path: str, counter: str):
    """kernel name -> [(counter value, grid size)] over its launches"""
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            acc[_short(r["Kernel_Name"])].append((float(r["Counter_Value"]), int(r.get("Grid_Size", 0) or 0)))
    return acc


def pmc(fetch_csv: str, write_csv: str, prefix: str = "gemm_bf16", which: str = "all") -> None:
    out = {"kernel_prefix": prefix, "launches_counted": which}
    key = "gemm" if prefix == "gemm_bf16" else "kernel"
    for counter, path in (("FETCH_SIZE", fetch_csv), ("WRITE_SIZE", write_csv)):
        acc = _per_kernel(path, counter)
        copies = [v for k, vals in acc.items() if "copy" in k.lower() or "Copy" in k for v, _ in vals]
        big = [v for v in copies if v > 0.75 * max(copies)]         # the 1 GiB calibration copies (a dtype-converting
                                                                   # copy of a 0.5 GiB tensor reads half as much)
        per_unit = GIB / (sum(big) / len(big))                      # bytes per counter unit
        sel = [(v, g) for k, vals in acc.items() if k.startswith(prefix) for v, g in vals]
        if which == "largest":
            gmax = max(g for _, g in sel)
            sel = [(v, g) for v, g in sel if g == gmax]
        vals = [v for v, _ in sel]
        out[counter] = {"calibration_copies": len(big), "bytes_per_counter_unit": per_unit,
                        key + "_launches": len(vals), key + "_bytes_per_launch": per_unit * sum(vals) / len(vals)}
    out["hbm_bytes_per_launch"] = out["FETCH_SIZE"][key + "_bytes_per_launch"] + out["WRITE_SIZE"][key + "_bytes_per_launch"]
    print(json.dumps(out, indent=1))


def counters(*paths: str) -> None:
    def fam(n):   # GEMM kernels per instantiation (tile and operand layouts), the others per name
        n = _short(n)
        return n if n.startswith("gemm_bf16") else n.split("<")[0]
    for path in paths:
        acc = collections.defaultdict(lambda: collections.defaultdict(float))
        launches = collections.defaultdict(set)
        for r in csv.DictReader(open(path)):
            k = fam(r["Kernel_Name"])
            if not (k.startswith("gemm_bf16") or k.startswith("attn_")):
                continue
            acc[k][r["Counter_Name"]] += float(r["Counter_Value"])
            launches[k].add(r["Dispatch_Id"])
        names = sorted({c for v in acc.values() for c in v})
        print("| kernel family | launches | " + " | ".join("`%s`" % c for c in names) + " |")
        print("|---|---|" + "---|" * len(names))
        for k in sorted(acc):
            v = acc[k]
            cells = []
            for c in names:
                cell = "%.4g" % v[c]
                for base in ("SQ_BUSY_CU_CYCLES", "SQ_WAVE_CYCLES"):
                    if base in v and c != base and v[base] > 0 and not c.startswith("SQ_INSTS") and c != "SQ_WAVES" \
                            and not (base == "SQ_WAVE_CYCLES" and "SQ_BUSY_CU_CYCLES" in v and not c.startswith("SQ_WAIT")):
                        cell += " (%.1f %% of %s)" % (100.0 * v[c] / v[base], base.replace("SQ_", "").lower())
                        break
                cells.append(cell)
            print("| `%s` | %d | " % (k, len(launches[k])) + " | ".join(cells) + " |")
        print()


def _durations(path: str):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        acc[_short(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    return acc


def durations(path: str, prefix: str, nbytes: str = "0") -> None:
    acc = _durations(path)
    v = sorted(x for k, vals in acc.items() if k.startswith(prefix) for x in vals)
    out = {"kernel_prefix": prefix, "launches": len(v), "avg_us": round(sum(v) / len(v), 2),
           "median_us": round(v[len(v) // 2], 2), "min_us": round(v[0], 2)}
    if float(nbytes) > 0:
        out["bytes_per_launch"] = float(nbytes)
        out["GBps_at_median"] = round(float(nbytes) / out["median_us"] / 1e3, 1)
        out["frac_of_8TBps_at_median"] = round(float(nbytes) / out["median_us"] / 1e3 / 8000.0, 3)
    print(json.dumps(out))


def streaming(path: str, tokens: str, d_model: str, d_ffn: str) -> None:
    T, d, f = int(tokens), int(d_model), int(d_ffn)
    acc = _durations(path)
    # algorithmic bytes per launch (bf16 tensors): what the kernel has to read and write once
    table = [("ln_fwd_kernel<unsigned short, 8, false", "LayerNorm forward", 4.0 * T * d, "x in, y out"),
             ("ln_fwd_kernel<unsigned short, 8, true", "LayerNorm forward, int8 input decoded", (1.0625 + 4.0) * T * d,
              "codes + scales in, x and y out"),
             ("ln_bwd_kernel<unsigned short, 2, false", "LayerNorm backward", 8.0 * T * d, "dy, x, residual gradient in, dx out"),
             ("ln_bwd_kernel<unsigned short, 2, true", "LayerNorm backward, int8 output encoded", (6.0 + 1.0625) * T * d,
              "dy, x, residual gradient in, codes + scales out"),
             ("colsum_partial_kernel", "bias-gradient column sums (four widths, average)", 2.0 * T * (5 * d + f) / 4,
              "gradient tensor in"),
             ("swarm::codec_encode_kernel", "codec encode", 3.0625 * T * d, "x in, codes + scales out"),
             ("swarm::codec_decode_kernel", "codec decode", 3.0625 * T * d, "codes + scales in, x out"),
             ("attn_delta_kernel", "attention backward row sums", 4.0 * T * d, "o, do in")]
    print("| kernel | what | launches | median us | algorithmic bytes per launch | GB/s | of 8 TB/s |")
    print("|---|---|---|---|---|---|---|")
    for prefix, what, nbytes, note in table:
        v = sorted(x for k, vals in acc.items() if k.startswith(prefix) for x in vals)
        if not v:
            continue
        med = v[len(v) // 2]
        print("| `%s` | %s (%s) | %d | %.1f | %.4g | %.0f | %.2f |" % (prefix.split("<")[0], what, note, len(v), med, nbytes,
                                                                 nbytes / med / 1e3, nbytes / med / 1e3 / 8000.0))


if __name__ == "__main__":
    {"stats": stats, "pmc": pmc, "counters": counters, "durations": durations,
     "streaming": streaming}[sys.argv[1]](*sys.argv[2:])
