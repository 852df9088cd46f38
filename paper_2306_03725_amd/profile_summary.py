"""Turns rocprofv3 output into the short text tables kept under profiles/.

  python -m paper_2306_03725_amd.profile_summary kernels RUN_results.db
      per-kernel calls / total / average / min / max duration from the rocpd database that
      `rocprofv3 --kernel-trace --stats -d DIR -o RUN -- python3 bench.py ...` writes

  python -m paper_2306_03725_amd.profile_summary bytes FETCH_counter_collection.csv WRITE_counter_collection.csv
      HBM-side KiB per launch of every kernel from two counter runs
      `rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR -o F -- python3 bench.py ... --calibrate-copy`
      (and the same with WRITE_SIZE), each scaled by what the same counter reads for the plain 1 GiB device
      copy that --calibrate-copy runs (2^20 KiB read, 2^20 KiB written)

Reads files only; runs nothing on a GPU.
"""
import collections
import csv
import re
import sqlite3
import sys

COPY_KERNEL = "__amd_rocclr_copyBuffer"     # the runtime's device-to-device copy
COPY_KIB = 1048576.0                        # it moves 2^30 bytes each way


def short(name, width=70):
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    return re.sub(r"\(.*", "", name)[:width]


def kernels(db_path, out=sys.stdout):
    cur = sqlite3.connect(db_path).cursor()
    rows = list(cur.execute("select name, count(*), sum(duration), avg(duration), min(duration), max(duration) "
                            "from kernels group by name order by sum(duration) desc"))
    total = sum(r[2] for r in rows) or 1
    out.write("%-72s %6s %11s %10s %10s %10s %6s\n" % ("kernel", "calls", "total_ms", "avg_us", "min_us", "max_us", "pct"))
    for name, calls, tot, avg, lo, hi in rows:
        out.write("%-72s %6d %11.3f %10.1f %10.1f %10.1f %6.2f\n"
                  % (short(name), calls, tot / 1e6, avg / 1e3, lo / 1e3, hi / 1e3, 100.0 * tot / total))


def _counter(path):
    per = collections.defaultdict(list)
    with open(path) as fh:
        for r in csv.DictReader(fh):
            per[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return per


def hbm_bytes(fetch_csv, write_csv, out=sys.stdout):
    fetch, write = _counter(fetch_csv), _counter(write_csv)
    if COPY_KERNEL not in fetch or COPY_KERNEL not in write:
        raise SystemExit("no %s launch in the counter files: run bench.py with --calibrate-copy" % COPY_KERNEL)
    sf, sw = COPY_KIB / max(fetch[COPY_KERNEL]), COPY_KIB / max(write[COPY_KERNEL])
    out.write("# calibration: the 1 GiB device copy reads FETCH_SIZE=%.1f, WRITE_SIZE=%.1f  =>  FETCH x%.3f, WRITE x%.3f\n"
              % (max(fetch[COPY_KERNEL]), max(write[COPY_KERNEL]), sf, sw))
    out.write("%-72s %6s %16s %16s %18s\n" % ("kernel", "n", "fetch KiB/launch", "write KiB/launch", "scaled MiB/launch"))

    def mean(v):
        return sum(v) / len(v) if v else 0.0
    for name in sorted(fetch, key=lambda n: -mean(fetch[n]) * len(fetch[n])):
        if "at::native" in name or "rocclr" in name:
            continue
        f, w = mean(fetch[name]), mean(write.get(name, []))
        out.write("%-72s %6d %16.1f %16.1f %18.1f\n" % (name, len(fetch[name]), f, w, (f * sf + w * sw) / 1024.0))


def main(argv):
    if len(argv) == 3 and argv[1] == "kernels":
        kernels(argv[2])
    elif len(argv) == 4 and argv[1] == "bytes":
        hbm_bytes(argv[2], argv[3])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv)
