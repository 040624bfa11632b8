"""Per-kernel hardware counters from a rocprofv3 --pmc run, as the short table kept under profiles/.

  python -m paper_1903_12650_amd.counter_summary <counter_collection.csv> "<command that made it>"

One line per kernel of the library (template arguments kept, so the tile shape is visible): dispatches, and the
mean of every collected counter per dispatch.  When SQ_VALU_MFMA_BUSY_CYCLES and GRBM_GUI_ACTIVE are both there,
also the matrix-core utilisation 100 * SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 * 1024): the counters are
summed over the chip (GRBM_GUI_ACTIVE over its 8 XCDs, SQ_* over 32 shader arrays), MFMA busy cycles over 1,024 SIMDs;
with SQ_BUSY_CYCLES / 32 in place of GRBM_GUI_ACTIVE / 8 the same ratio over the cycles the shader arrays were busy;
SQ_INSTS_VALU_MFMA_MOPS_BF16 * 512 is the bf16 flop count (one unit = 512 flop).
"""
import collections
import csv
import re
import sys


def main():
    path, cmd = sys.argv[1], sys.argv[2]
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    seen = collections.defaultdict(set)
    for r in csv.DictReader(open(path)):
        k = r["Kernel_Name"]
        if "rn50::" not in k:
            continue
        k = re.sub(r"\(.*$", "", k).replace("void rn50::", "").replace("unsigned short", "bf16")
        agg[k][r["Counter_Name"]] += float(r["Counter_Value"])
        seen[k].add(r["Dispatch_Id"])
    print("command:", cmd)
    for k in sorted(agg):
        n = len(seen[k])
        c = {name: v / n for name, v in agg[k].items()}
        print("%s   dispatches %d" % (k, n))
        for name in sorted(c):
            print("    %-34s %16.0f per dispatch" % (name, c[name]))
        busy = c.get("SQ_VALU_MFMA_BUSY_CYCLES")
        if busy is not None and c.get("GRBM_GUI_ACTIVE"):
            print("    matrix-core utilisation, MFMA busy / (GRBM_GUI_ACTIVE / 8 XCDs * 1024 SIMDs): %.1f %%"
                  % (100.0 * busy / (c["GRBM_GUI_ACTIVE"] / 8 * 1024)))
        if busy is not None and c.get("SQ_BUSY_CYCLES"):
            print("    while the shader arrays were busy, MFMA busy / (SQ_BUSY_CYCLES / 32 arrays * 1024 SIMDs): %.1f %%"
                  % (100.0 * busy / (c["SQ_BUSY_CYCLES"] / 32 * 1024)))
        if c.get("SQ_LDS_BANK_CONFLICT") is not None and c.get("SQ_LDS_IDX_ACTIVE"):
            print("    LDS cycles lost to bank conflicts: %.1f %%" % (100.0 * c["SQ_LDS_BANK_CONFLICT"] / c["SQ_LDS_IDX_ACTIVE"]))
        if c.get("SQ_INSTS_VALU_MFMA_MOPS_BF16"):
            print("    bf16 matrix flop: %.3f G" % (c["SQ_INSTS_VALU_MFMA_MOPS_BF16"] * 512 / 1e9))


if __name__ == "__main__":
    main()
