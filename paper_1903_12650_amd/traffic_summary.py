"""HBM traffic per launch from rocprofv3 counter files, scaled by a copy of known size.

  python -m paper_1903_12650_amd.traffic_summary <FETCH counter_collection.csv> <WRITE counter_collection.csv> \
         <bytes the calibration copy reads (= writes)> <steps profiled> "<command>"

Each CSV comes from one `rocprofv3 --pmc FETCH_SIZE` (resp. WRITE_SIZE) run of
`bench.py --calibration-copy`.  The calibration dispatch is the device copy bench.py makes of the float
master arena (the largest dispatch of the runtime's buffer-copy kernel); the factor bytes/counter it gives
is applied to every kernel of the library, grouped by the step's launch tags.
"""
import collections
import csv
import re
import sys

TAGS = [("conv_fwd", r"igemm_kernel<[^,]+(, \d+){4}, 0,"), ("conv_dgrad", r"igemm_kernel<[^,]+(, \d+){4}, 1,"), ("conv_wgrad", r"wgrad(3x3)?_kernel"),
        ("conv_wgrad_reduce", r"splitk_reduce"), ("bn_finalize", r"bn_finalize_kernel"), ("bn_apply", r"bn_apply_kernel"),
        ("bn_bwd_reduce", r"bn_bwd_reduce"), ("bn_bwd_finalize", r"bn_bwd_finalize"), ("bn_bwd_apply", r"bn_bwd_apply"),
        ("lars_norms", r"lars_norms"), ("lars_apply", r"lars_apply")]


def read(path, counter):
    per_kernel = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        per_kernel[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return per_kernel


def factor(per_kernel, known_bytes):
    cands = [(k, v) for k, v in per_kernel.items() if "copybuffer" in k.lower()]
    if not cands:
        cands = [(k, v) for k, v in per_kernel.items() if "copy" in k.lower() and "rn50" not in k]
    # the calibration copy is the largest copy dispatch of the run
    best = max(((max(v), k) for k, v in cands), default=None)
    if best is None:
        raise SystemExit("no copy dispatch found")
    return known_bytes / best[0], best[1], best[0]


def main():
    fpath, wpath, known, steps, cmd = sys.argv[1], sys.argv[2], float(sys.argv[3]), int(sys.argv[4]), sys.argv[5]
    F, W = read(fpath, "FETCH_SIZE"), read(wpath, "WRITE_SIZE")
    ff, fk, fv = factor(F, known)
    wf, wk, wv = factor(W, known)
    print("command:", cmd)
    print(f"calibration copy ({known:.0f} bytes each way): FETCH_SIZE {fv:.0f} -> {ff:.1f} bytes/unit [{fk[:40]}], "
          f"WRITE_SIZE {wv:.0f} -> {wf:.1f} bytes/unit [{wk[:40]}]")
    print("%-20s %9s %16s %16s %16s" % ("launch tag", "launches", "fetch MB/launch", "write MB/launch", "total MB/launch"))
    for tag, pat in TAGS:
        f = [v for k, vs in F.items() if re.search(pat, k) for v in vs]
        w = [v for k, vs in W.items() if re.search(pat, k) for v in vs]
        if not f:
            continue
        fb, wb = sum(f) * ff / len(f), sum(w) * wf / max(len(w), 1)
        print("%-20s %9d %16.2f %16.2f %16.2f" % (tag, len(f) // steps, fb / 1e6, wb / 1e6, (fb + wb) / 1e6))


if __name__ == "__main__":
    main()
