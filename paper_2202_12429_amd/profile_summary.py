"""Text summaries of rocprofv3 runs of this library's kernels (the files under profiles/), and the link between such
a summary and the kernel sources it was measured on.

    python -m paper_2202_12429_amd.profile_summary stats <dir> <prefix>            # --kernel-trace --stats run
    python -m paper_2202_12429_amd.profile_summary pmc <dir>                        # FETCH_SIZE + WRITE_SIZE runs

Both print the summary to stdout; its first lines name the digest of the kernel sources (csrc/ and the C header), so
that a reader of the numbers, bench.py among them, can tell whether the kernels have changed since.
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import os
import re
import statistics
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
DIGEST_TAG = "kernel-sources-sha256:"
TRAFFIC_TAG = "traffic-bytes-per-launch"


def kernel_source_digest() -> str:
    """First 16 hex digits of the SHA-256 over the HIP sources and the C header, in name order."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")) + glob.glob(os.path.join(HERE, "csrc", "*.h")))
    files.append(os.path.join(ROOT, "include", "bagpipe.h"))
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def short_kernel_name(full: str) -> str:
    n = full.replace("(anonymous namespace)::", "")
    m = re.search(r"bp::([a-z_0-9]+)(<[^(]*>)?", n)
    if not m:
        return ""
    key = m.group(1) + (m.group(2) or "")
    return key.replace("unsigned long", "u64").replace("unsigned int", "u32").replace("bp::", "")


def stats_summary(directory: str, prefix: str) -> str:
    """Per-kernel call counts and durations from <dir>/**/<prefix>_kernel_trace.csv (rocprofv3 --kernel-trace)."""
    paths = glob.glob(os.path.join(directory, "**", f"{prefix}_kernel_trace.csv"), recursive=True)
    if not paths:
        raise SystemExit(f"no {prefix}_kernel_trace.csv under {directory}")
    dur = collections.defaultdict(list)
    for r in csv.DictReader(open(paths[0])):
        k = short_kernel_name(r["Kernel_Name"])
        if k:
            dur[k].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    lines = [f"{DIGEST_TAG} {kernel_source_digest()}",
             f"{'kernel':74s} {'calls':>7s} {'avg_us':>9s} {'median_us':>9s} {'min_us':>9s} {'max_us':>9s} {'total_ms':>9s}"]
    for k in sorted(dur, key=lambda k: -sum(dur[k])):
        d = dur[k]
        lines.append(f"{k[:72]:74s} {len(d):7d} {statistics.mean(d):9.2f} {statistics.median(d):9.2f} {min(d):9.2f} "
                     f"{max(d):9.2f} {sum(d) / 1e3:9.3f}")
    return "\n".join(lines)


def pmc_summary(directory: str) -> str:
    """HBM-side bytes per launch from <dir>/**/pmc_FETCH_SIZE_counter_collection.csv and ..._WRITE_SIZE_...: counter
    values are KiB per dispatch; each counter is scaled by what it reads for the plain copy kernel of known size."""
    def load(counter):
        paths = glob.glob(os.path.join(directory, "**", f"pmc_{counter}_counter_collection.csv"), recursive=True)
        if not paths:
            raise SystemExit(f"no pmc_{counter}_counter_collection.csv under {directory}")
        out = collections.defaultdict(list)
        for r in csv.DictReader(open(paths[0])):
            k = short_kernel_name(r["Kernel_Name"])
            if k:
                out[k].append(float(r["Counter_Value"]))
        return out
    F, W = load("FETCH_SIZE"), load("WRITE_SIZE")
    true_kib = 2 ** 30 / 1024
    cf, cw = statistics.mean(F["copy_calibration_kernel"]), statistics.mean(W["copy_calibration_kernel"])
    kf, kw = true_kib / cf, true_kib / cw
    lines = [f"{DIGEST_TAG} {kernel_source_digest()}",
             f"copy_calibration_kernel (1 GiB read, 1 GiB written): FETCH_SIZE {cf:.1f}  WRITE_SIZE {cw:.1f}  "
             f"(true: {true_kib:.0f} KiB each)",
             f"scale factors: fetch x{kf:.4f}, write x{kw:.4f}",
             f"{'kernel':62s} {'n':>5s} {'FETCH_SIZE':>12s} {'WRITE_SIZE':>12s} {'fetch MB':>10s} {'write MB':>10s} {'total MB':>10s}"]
    traffic = []
    for k in sorted(F, key=lambda k: -sum(F[k])):
        f, w = statistics.mean(F[k]), statistics.mean(W.get(k, [0.0]))
        fm, wm = f * kf * 1024 / 1e6, w * kw * 1024 / 1e6
        lines.append(f"{k[:60]:62s} {len(F[k]):5d} {f:12.1f} {w:12.1f} {fm:10.2f} {wm:10.2f} {fm + wm:10.2f}")
        traffic.append(f"{TRAFFIC_TAG} {k.split('<')[0]} {(fm + wm) * 1e6:.0f}")
    return "\n".join(lines + [""] + traffic)


def read_traffic(path: str):
    """(digest, {kernel name without template arguments: bytes per launch}) of a pmc summary; (None, {}) if absent."""
    digest, traffic = None, {}
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(DIGEST_TAG):
                    digest = line.split()[1]
                elif line.startswith(TRAFFIC_TAG):
                    _, name, val = line.split()
                    traffic.setdefault(name, float(val))
    except OSError:
        pass
    return digest, traffic


if __name__ == "__main__":
    if len(sys.argv) >= 4 and sys.argv[1] == "stats":
        print(stats_summary(sys.argv[2], sys.argv[3]))
    elif len(sys.argv) >= 3 and sys.argv[1] == "pmc":
        print(pmc_summary(sys.argv[2]))
    else:
        raise SystemExit(__doc__)
