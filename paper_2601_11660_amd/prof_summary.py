"""Turns rocprofv3 CSV output into the short text tables kept under profiles/.

    python -m paper_2601_11660_amd.prof_summary stats   <dir>/<prefix>_kernel_stats.csv
    python -m paper_2601_11660_amd.prof_summary traffic <fetch>_counter_collection.csv \
                                                        <write>_counter_collection.csv
    python -m paper_2601_11660_amd.prof_summary counters <file>_counter_collection.csv [...]
    python -m paper_2601_11660_amd.prof_summary ramp <bench --ramp output> [<SQ_BUSY_CU_CYCLES csv>]

`traffic` expects the two counter passes of `bench.py --calibrate-copy` (FETCH_SIZE, then
WRITE_SIZE): the three plain 256 MiB device copies at the end of that run give the scale factor
of each counter, and the table lists HBM bytes per launch for every kernel of the library,
together with the digest of the kernel sources it was measured on (bench.py drops the figure
when the sources have changed since).
"""
import collections
import csv
import hashlib
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
COPY_KIB = 262144.0      # bytes moved each way by one calibration copy, in KiB


def csrc_digest():
    h = hashlib.sha256()
    d = os.path.join(HERE, "csrc")
    for name in sorted(os.listdir(d)):
        h.update(name.encode())
        with open(os.path.join(d, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def short(name):
    """mbu::conv_mfma_block_kernel<4, 1, ...>(args) -> conv_mfma_block_kernel<4, 1, ...>"""
    name = name.replace("void ", "")
    depth = 0
    for i, ch in enumerate(name):
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            name = name[:i]
            break
    return name.replace("mbu::", "")


def base(name):
    return short(name).split("<")[0]


def stats(path):
    rows = list(csv.DictReader(open(path)))
    print("| kernel | calls | total us | avg us | min us | max us | % |")
    print("|---|---|---|---|---|---|---|")
    conv_calls = conv_ns = 0
    for r in rows:
        ns = float(r["TotalDurationNs"])
        print(f"| {short(r['Name'])} | {r['Calls']} | {ns / 1e3:.1f} | {float(r['AverageNs']) / 1e3:.2f} | "
              f"{float(r['MinNs']) / 1e3:.2f} | {float(r['MaxNs']) / 1e3:.2f} | {float(r['Percentage']):.2f} |")
        if base(r["Name"]).startswith("conv_mfma"):
            conv_calls += int(r["Calls"])
            conv_ns += ns
    if conv_calls:
        print(f"\nconv kernels together: {conv_calls} launches, {conv_ns / 1e3:.1f} us, "
              f"average {conv_ns / 1e3 / conv_calls:.2f} us per launch")


def read_counter(path, counter):
    per = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            per[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return per


def traffic(fetch_csv, write_csv):
    f = read_counter(fetch_csv, "FETCH_SIZE")
    w = read_counter(write_csv, "WRITE_SIZE")

    def copies(per):
        for k, v in per.items():
            if "copyBuffer" in k:
                return v[-3:]
        raise SystemExit("no calibration copy in the counter file (run bench.py --calibrate-copy)")

    cf, cw = copies(f), copies(w)
    sf = COPY_KIB / (sum(cf) / len(cf))
    sw = COPY_KIB / (sum(cw) / len(cw))
    print(f"calibration copies (256 MiB each way), KiB per dispatch: FETCH_SIZE {cf} -> scale {sf:.3f}; "
          f"WRITE_SIZE {cw} -> scale {sw:.3f}\n")
    print("| kernel | launches | fetched MB / launch | written MB / launch | total bytes / launch |")
    print("|---|---|---|---|---|")
    tot = {}
    for k in sorted(f, key=lambda k: -sum(f[k])):
        if "mbu::" not in k or k not in w:
            continue
        fb = sum(f[k]) / len(f[k]) * sf * 1024
        wb = sum(w[k]) / len(w[k]) * sw * 1024
        print(f"| {short(k)} | {len(f[k])} | {fb / 1e6:.2f} | {wb / 1e6:.2f} | {fb + wb:.0f} |")
        b = base(k)
        n0, t0 = tot.get(b, (0, 0.0))
        tot[b] = (n0 + len(f[k]), t0 + (fb + wb) * len(f[k]))
    print()
    print(f"csrc_sha256: {csrc_digest()}")
    for b, (n, t) in sorted(tot.items()):
        print(f"traffic_bytes_per_launch[{b}]: {t / n:.0f}")


def counters(paths):
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    for p in paths:
        for r in csv.DictReader(open(p)):
            if "mbu::" in r["Kernel_Name"]:
                per[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    names = sorted({c for k in per for c in per[k]})
    print("| kernel | launches | " + " | ".join(names) + " |")
    print("|---|---|" + "---|" * len(names))
    for k in sorted(per):
        n = max(len(v) for v in per[k].values())
        cells = [f"{sum(per[k][c]) / len(per[k][c]):.0f}" if per[k][c] else "-" for c in names]
        print(f"| {k} | {n} | " + " | ".join(cells) + " |")


def ramp(json_path, pmc_csv=None):
    """Pass time against pass index after an idle period (bench.py --ramp), in blocks of ten
    passes; with a counter file of the same command, the shader clock of each block =
    SQ_BUSY_CU_CYCLES / 256 compute units / dispatch duration over the block's forward-pass
    dispatches."""
    import json
    ms = json.load(open(json_path))["ramp_ms_per_pass"]
    clock = None
    if pmc_csv:
        rows = [r for r in csv.DictReader(open(pmc_csv))
                if r["Counter_Name"] == "SQ_BUSY_CU_CYCLES" and "mbu::" in r["Kernel_Name"]
                and "pack" not in r["Kernel_Name"] and "count_kept" not in r["Kernel_Name"]]
        rows.sort(key=lambda r: int(r["Dispatch_Id"]))
        per_pass = 20
        rows = rows[3 * per_pass:]                     # the three passes before the idle period
        clock = []
        for b in range(len(ms) // 10):
            blk = rows[b * 10 * per_pass:(b + 1) * 10 * per_pass]
            if len(blk) < 10 * per_pass:
                break
            cyc = sum(float(r["Counter_Value"]) for r in blk) / 256.0
            ns = sum(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in blk)
            clock.append(cyc / ns)
    print("| passes | mean ms per pass | frames/s |" + (" shader clock GHz (counter pass) |" if clock else ""))
    print("|---|---|---|" + ("---|" if clock else ""))
    for b in range(len(ms) // 10):
        m = sum(ms[b * 10:(b + 1) * 10]) / 10
        extra = f" {clock[b]:.2f} |" if clock and b < len(clock) else (" - |" if clock else "")
        print(f"| {b * 10 + 1}-{b * 10 + 10} | {m:.4f} | {1e3 / m:.0f} |" + extra)


if __name__ == "__main__":
    mode = sys.argv[1]
    if mode == "stats":
        stats(sys.argv[2])
    elif mode == "traffic":
        traffic(sys.argv[2], sys.argv[3])
    elif mode == "counters":
        counters(sys.argv[2:])
    elif mode == "ramp":
        ramp(sys.argv[2], sys.argv[3] if len(sys.argv) > 3 else None)
    else:
        raise SystemExit(__doc__)
