"""Condenses rocprofv3 CSV output of a bench.py run into a short text summary.

Usage (after the profiler runs named in the summary's header):
    python profile_summary.py --workload 'configs[1]' --kernel range_kernel --bench-args='--config 1 ...' \
        --kernel-trace out/prof_kt --fetch out/prof_fetch --write out/prof_write \
        > profiles/range_kernel_config1.md

FETCH_SIZE and WRITE_SIZE are reported by rocprofv3 in KiB per dispatch.  Each
is scaled by what the same counter reads for a device-to-device copy of known
size in the same run (bench.py --copy-calibration copies 1 GiB three times):
factor = 2^20 KiB / counter value of that copy.  The line that starts with
`traffic_bytes_per_launch` is the one bench.py looks up; it carries a hash of
the kernel sources so that a stale figure is never reported.
"""
import argparse
import csv
import glob
import hashlib
import os
import statistics

ROOT = os.path.dirname(os.path.abspath(__file__))
COPY_KIB = float(1 << 20)
# the sources bench.py hashes for each main kernel
KERNEL_SOURCES = {
    "range_kernel": ("attn_range.hip", "attn_tile.h", "kernels.h"),
    "split_kernel": ("attn_split.hip", "attn_tile.h", "kernels.h"),
    "prefill_kernel": ("attn_prefill.hip", "attn_tile.h", "kernels.h"),
}


def source_hash(kernel):
    h = hashlib.sha256()
    for s in KERNEL_SOURCES[kernel]:
        h.update(open(os.path.join(ROOT, "paper_2508_11553_amd", "csrc", s), "rb").read())
    return h.hexdigest()[:16]


def one(pattern):
    hits = sorted(glob.glob(pattern))
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return hits[0]


def counters(directory, counter):
    """{kernel name: [values per dispatch]} for one counter."""
    out = {}
    with open(one(os.path.join(directory, "*counter_collection.csv"))) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                out.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return out


def calibration(values_by_kernel):
    """Scale factor from the large device copies (the three biggest copyBuffer dispatches)."""
    vals = sorted(values_by_kernel.get("__amd_rocclr_copyBuffer", []))[-3:]
    if not vals or min(vals) <= 0:
        raise SystemExit("no calibration copy found: run bench.py with --copy-calibration")
    return COPY_KIB / statistics.mean(vals), vals


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--kernel", default="range_kernel", choices=sorted(KERNEL_SOURCES),
                    help="the main kernel of this workload (its traffic line is what bench.py looks up)")
    ap.add_argument("--kernel-trace", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--mfma", default=None, help="optional fourth run: --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES")
    ap.add_argument("--bench-args", required=True,
                    help="the arguments bench.py was given in the kernel-trace run, --config N included (for the header)")
    ap.add_argument("--pmc-bench-args", required=True, help="the arguments of the counter runs")
    a = ap.parse_args()

    print(f"# rocprofv3 summary: bench.py, workload {a.workload}\n")
    print("Commands (each from the repository root, after `cd /tmp && export TMPDIR=/tmp`):\n")
    print(f"    rocprofv3 --kernel-trace --stats --output-format csv -d {a.kernel_trace} -o run -- python3 bench.py {a.bench_args}")
    print(f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d {a.fetch} -o run -- python3 bench.py {a.pmc_bench_args}")
    print(f"    rocprofv3 --pmc WRITE_SIZE --output-format csv -d {a.write} -o run -- python3 bench.py {a.pmc_bench_args}")
    if a.mfma:
        print(f"    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES --output-format csv -d {a.mfma} -o run -- "
              f"python3 bench.py {a.pmc_bench_args}")
    print(f"    python profile_summary.py --workload '{a.workload}' --kernel {a.kernel} --bench-args='{a.bench_args}' "
          f"--pmc-bench-args='{a.pmc_bench_args}' --kernel-trace {a.kernel_trace} "
          f"--fetch {a.fetch} --write {a.write}" + (f" --mfma {a.mfma}" if a.mfma else "") + "\n")

    print("## Kernel durations (--kernel-trace --stats)\n")
    print("| kernel | calls | avg us | min us | max us | % of GPU time |")
    print("|---|---|---|---|---|---|")
    with open(one(os.path.join(a.kernel_trace, "*kernel_stats.csv"))) as f:
        for r in csv.DictReader(f):
            name = r["Name"]
            if len(name) > 70:
                name = name[:67] + "..."
            print(f"| `{name}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.2f} | {float(r['MinNs']) / 1e3:.2f} | "
                  f"{float(r['MaxNs']) / 1e3:.2f} | {float(r['Percentage']):.2f} |")

    fetch, write = counters(a.fetch, "FETCH_SIZE"), counters(a.write, "WRITE_SIZE")
    ff, fvals = calibration(fetch)
    wf, wvals = calibration(write)
    print("\n## HBM traffic counters (--pmc, KiB per dispatch)\n")
    print(f"Calibration: a 1 GiB device copy reads FETCH_SIZE = {statistics.mean(fvals):.0f} and WRITE_SIZE = "
          f"{statistics.mean(wvals):.0f}; factors {ff:.4f} (fetch) and {wf:.4f} (write).\n")
    print("| kernel | dispatches | FETCH_SIZE raw | WRITE_SIZE raw | read MB scaled | written MB scaled |")
    print("|---|---|---|---|---|---|")
    total = {}
    for name in fetch:
        if name not in write or name.startswith("__amd") or "at::native" in name:
            continue
        fr, wr = statistics.mean(fetch[name]), statistics.mean(write[name])
        rd, wrb = fr * ff * 1024, wr * wf * 1024
        total[name] = rd + wrb
        short = name if len(name) <= 70 else name[:67] + "..."
        print(f"| `{short}` | {len(fetch[name])} | {fr:.1f} | {wr:.1f} | {rd / 1e6:.2f} | {wrb / 1e6:.2f} |")
    if a.mfma:
        busy, cu = counters(a.mfma, "SQ_VALU_MFMA_BUSY_CYCLES"), counters(a.mfma, "SQ_BUSY_CU_CYCLES")
        print("\n## Matrix-core utilisation (--pmc)\n")
        print("MFMA busy cycles summed over the SIMDs, against 4 SIMDs x the cycles a CU was busy.\n")
        print("| kernel | SQ_VALU_MFMA_BUSY_CYCLES | SQ_BUSY_CU_CYCLES | MFMA busy, % of SIMD cycles |")
        print("|---|---|---|---|")
        for name in busy:
            if name not in cu or a.kernel not in name:
                continue
            bz, cz = statistics.mean(busy[name]), statistics.mean(cu[name])
            short = name if len(name) <= 70 else name[:67] + "..."
            print(f"| `{short}` | {bz:.3g} | {cz:.3g} | {100.0 * bz / (4.0 * cz):.1f} |")
    print()
    tag = source_hash(a.kernel)
    for name, t in total.items():
        if a.kernel in name and "Lb1" not in name and ", true>" not in name:   # not the probe instantiation
            print(f"traffic_bytes_per_launch workload={a.workload} source_sha256={tag} kernel={name.split('(')[0].replace('void ', '').replace(' ', '')} value={t:.0f}")


if __name__ == "__main__":
    main()
