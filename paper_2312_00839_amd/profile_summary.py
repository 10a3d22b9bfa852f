"""Turns rocprofv3's CSV output for a bench.py run into the short text summaries kept under profiles/.

    python -m paper_2312_00839_amd.profile_summary traffic --fetch F.csv --write W.csv --kernel step_predict_kernel \
        --variant fused-config5-adamw-local-gf32-hbf16 --algorithmic-bytes 22146662400
    python -m paper_2312_00839_amd.profile_summary trace --stats kt_kernel_stats.csv --kernel step_predict_kernel \
        --variant ... --algorithmic-bytes ...

`traffic`: FETCH_SIZE and WRITE_SIZE (KiB per dispatch, one counter per rocprofv3 --pmc run) averaged over the
dispatches of the kernel, each scaled by what the same counter reads for the library's plain copy kernel
(`probe_copy_kernel`, which bench.py runs on 4 GiB in the same process: it reads 4 GiB and writes 4 GiB).
`trace`: the kernel's row of `rocprofv3 --kernel-trace --stats`.
Both print a `kernel_source_sha256` line: bench.py quotes a summary's traffic figure only while the kernel source
in the tree still has that fingerprint.
"""
import argparse
import csv
import hashlib
import os
import sys

CSRC = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
COPY_KERNEL = "probe_copy_kernel"
COPY_BYTES = 4 << 30


def kernel_source_sha256():
    """Fingerprint of the kernels' source files."""
    h = hashlib.sha256()
    for name in ("step_predict_kernels.hip", "po_internal.h"):
        with open(os.path.join(CSRC, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def _counter_means(path, counter):
    """{kernel name: (mean value, dispatches)} of one counter in a rocprofv3 counter_collection CSV."""
    acc = {}
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            if row["Counter_Name"] != counter:
                continue
            a = acc.setdefault(row["Kernel_Name"], [0.0, 0])
            a[0] += float(row["Counter_Value"])
            a[1] += 1
    return {k: (v[0] / v[1], v[1]) for k, v in acc.items()}


def _pick(means, needle, what):
    hits = {k: v for k, v in means.items() if needle in k}
    if len(hits) != 1:
        sys.exit("%s: expected exactly one kernel matching %r, found %d: %s" % (what, needle, len(hits), sorted(hits)))
    return next(iter(hits.items()))


def traffic(args):
    out = []
    total = 0
    for counter, path in (("FETCH_SIZE", args.fetch), ("WRITE_SIZE", args.write)):
        means = _counter_means(path, counter)
        kname, (kval, kn) = _pick(means, args.kernel, counter)
        cname, (cval, cn) = _pick(means, COPY_KERNEL, counter)
        factor = (COPY_BYTES / 1024.0) / cval
        nbytes = kval * 1024.0 * factor
        total += nbytes
        out.append("  %-10s %s: %.1f KiB per dispatch over %d dispatches" % (counter, kname.replace("(anonymous namespace)::", "").replace("void ", "").split("(")[0], kval, kn))
        out.append("  %-10s %s (moves 4 GiB each way = 4194304 KiB): %.1f KiB over %d dispatches -> scale factor %.6f"
                   % (counter, COPY_KERNEL, cval, cn, factor))
        out.append("  %-10s scaled: %.0f bytes per launch" % (counter, nbytes))
    out.append("  total %.0f bytes per launch; algorithmic %d; ratio %.5f" % (total, args.algorithmic_bytes, total / args.algorithmic_bytes))
    out.append("traffic_bytes_per_launch variant=%s bytes=%d" % (args.variant, round(total)))
    out.append("kernel_source_sha256: %s" % kernel_source_sha256())
    print("\n".join(out))


def trace(args):
    rows = []
    with open(args.stats, newline="") as f:
        for row in csv.DictReader(f):
            if args.kernel in row["Name"]:
                rows.append(row)
    if len(rows) != 1:
        sys.exit("trace: expected exactly one kernel matching %r, found %d" % (args.kernel, len(rows)))
    r = rows[0]
    avg = float(r["AverageNs"])
    print("  %s" % r["Name"].replace("(anonymous namespace)::", "").replace("void ", "").split("(")[0])
    print("  calls %s  average %.1f us  min %.1f us  max %.1f us  stddev %.1f us"
          % (r["Calls"], avg / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, float(r["StdDev"]) / 1e3))
    gbps = args.algorithmic_bytes / avg
    print("  algorithmic %d bytes per launch / average duration = %.1f GB/s = %.4f of 8000 GB/s" % (args.algorithmic_bytes, gbps, gbps / 8000.0))
    print("kernel_trace_average_ns variant=%s ns=%.1f" % (args.variant, avg))
    print("kernel_source_sha256: %s" % kernel_source_sha256())


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("traffic")
    t.add_argument("--fetch", required=True)
    t.add_argument("--write", required=True)
    t.add_argument("--kernel", required=True)
    t.add_argument("--variant", required=True)
    t.add_argument("--algorithmic-bytes", type=int, required=True)
    t.set_defaults(fn=traffic)
    k = sub.add_parser("trace")
    k.add_argument("--stats", required=True)
    k.add_argument("--kernel", required=True)
    k.add_argument("--variant", required=True)
    k.add_argument("--algorithmic-bytes", type=int, required=True)
    k.set_defaults(fn=trace)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
