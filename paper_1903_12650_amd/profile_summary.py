"""Turn rocprofv3's <name>_kernel_stats.csv (from `rocprofv3 --kernel-trace --stats --output-format csv`)
into the short text table kept under profiles/.

  python -m paper_1903_12650_amd.profile_summary <kernel_stats.csv> <steps profiled> "<command that made it>"
"""
import csv
import re
import sys


def main():
    path, steps, cmd = sys.argv[1], int(sys.argv[2]), sys.argv[3]
    rows = list(csv.DictReader(open(path)))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print("command:", cmd)
    print(f"steps profiled (warm-up included): {steps}")
    print(f"total kernel time {total / 1e6:.3f} ms = {total / 1e6 / steps:.3f} ms per step over "
          f"{sum(int(r['Calls']) for r in rows)} launches ({sum(int(r['Calls']) for r in rows) / steps:.0f} per step)")
    print("%-64s %7s %10s %9s %9s %9s %6s" % ("kernel", "calls", "total_us", "avg_us", "min_us", "max_us", "%"))
    for r in rows:
        name = re.sub(r"\(.*$", "", r["Name"]).replace("void ", "").replace("unsigned short", "bf16")
        print("%-64s %7d %10.1f %9.2f %9.2f %9.2f %6.2f" % (name[:64], int(r["Calls"]), float(r["TotalDurationNs"]) / 1e3,
                                                          float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
                                                          float(r["MaxNs"]) / 1e3, float(r["Percentage"])))


if __name__ == "__main__":
    main()
