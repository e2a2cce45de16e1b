"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

Usage (after the rocprofv3 runs named in each summary's header):
    python -m paper_2401_09149_amd.profile_summary stats  <kernel_stats.csv> <out.md> "<command>"
    python -m paper_2401_09149_amd.profile_summary pmc    <out.md> "<command>" <counter_collection.csv> [...]
    python -m paper_2401_09149_amd.profile_summary traffic <fetch.csv> <write.csv> <out.json> <workload> "<command>"
"""
import collections
import csv
import json
import sys


def ours(kernel):
    return "attn_" in kernel or "sp_permute" in kernel or "linear_gemm" in kernel


def short(name):
    name = name.replace("(anonymous namespace)::", "").split("(")[0]
    return name.replace("void ", "").replace("ie::", "")


def stats(src, out, command):
    rows = list(csv.DictReader(open(src)))
    with open(out, "w") as f:
        f.write(f"# rocprofv3 --kernel-trace --stats\n\ncommand: `{command}`\n\n")
        f.write("| kernel | calls | avg ms | min ms | max ms | % of GPU time |\n|---|---|---|---|---|---|\n")
        for r in rows:
            f.write(f"| {short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']) / 1e6:.3f} | {float(r['MinNs']) / 1e6:.3f} | "
                    f"{float(r['MaxNs']) / 1e6:.3f} | {float(r['Percentage']):.2f} |\n")


def per_kernel(path, skip_first=1):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        agg[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    out = {}
    for k, cs in agg.items():
        out[k] = {c: (sum(v[skip_first:]) / len(v[skip_first:]) if len(v) > skip_first else v[-1]) for c, v in cs.items()}
    return out


def pmc(out, command, paths):
    merged = collections.defaultdict(dict)
    for pth in paths:
        for k, cs in per_kernel(pth).items():
            merged[k].update(cs)
    with open(out, "w") as f:
        f.write(f"# rocprofv3 --pmc (one run per counter group), mean per dispatch\n\ncommand: `{command}`\n\n")
        for k, cs in merged.items():
            if not ours(k):
                continue
            f.write(f"## {k}\n\n")
            for c, v in sorted(cs.items()):
                f.write(f"- {c}: {v:.4g}\n")
            f.write("\n")


def traffic(fetch_csv, write_csv, out, workload, command):
    """FETCH_SIZE / WRITE_SIZE are in KiB per dispatch up to a device-dependent factor; the factor
    is what a plain copy of 2^30 bytes reads in the same run."""
    fetch, write = per_kernel(fetch_csv), per_kernel(write_csv)

    def copy_value(table, counter):
        # the runtime's device-to-device copy kernel (torch's copy_ of a contiguous buffer); failing that,
        # the largest kernel that is not one of ours
        named = [cs[counter] for k, cs in table.items() if "copyBuffer" in k and counter in cs and cs[counter] > 2 ** 18]
        if named:
            return max(named)
        cands = [cs[counter] for k, cs in table.items() if not ours(k) and counter in cs and cs[counter] > 2 ** 18]
        return max(cands) if cands else None

    cf, cw = copy_value(fetch, "FETCH_SIZE"), copy_value(write, "WRITE_SIZE")
    kib = float(2 ** 20)
    sf = kib / cf if cf else 1.0   # true KiB per counted unit
    sw = kib / cw if cw else 1.0
    res = {"workload": workload, "command": command, "fetch_scale": sf, "write_scale": sw,
           "copy_fetch_counter": cf, "copy_write_counter": cw, "bytes_per_launch": {}, "detail": {}}
    groups = collections.defaultdict(list)   # instantiations of one kernel template share a name: mean over them
    for k in fetch:
        if not ours(k):
            continue
        fb = fetch[k].get("FETCH_SIZE", 0.0) * sf * 1024.0
        wb = write.get(k, {}).get("WRITE_SIZE", 0.0) * sw * 1024.0
        name = k.split("<")[0]
        if name == "attn_bwd_dkdv_kernel" and "true" in k:   # except the instantiation that also stores dS
            name += "_store_ds"
        groups[name].append((fb, wb))
    for name, vals in groups.items():
        fb = sum(v[0] for v in vals) / len(vals)
        wb = sum(v[1] for v in vals) / len(vals)
        res["bytes_per_launch"][name] = fb + wb
        res["detail"][name] = {"fetch_bytes": fb, "write_bytes": wb}
    with open(out, "w") as f:
        json.dump(res, f, indent=1)
        f.write("\n")


if __name__ == "__main__":
    mode = sys.argv[1]
    if mode == "stats":
        stats(sys.argv[2], sys.argv[3], sys.argv[4])
    elif mode == "pmc":
        pmc(sys.argv[2], sys.argv[3], sys.argv[4:])
    elif mode == "traffic":
        traffic(*sys.argv[2:7])
    else:
        raise SystemExit(__doc__)
