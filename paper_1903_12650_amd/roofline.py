"""Algorithmic cost model of the step's kernels (what the method itself must move or multiply,
independent of how the kernels are written) and the roofline record bench.py prints.

Per unit of work (elements are activation elements of the BN's tensor, bf16 = 2 bytes):
  conv_fwd / conv_dgrad  2*M*N*K flop;  bytes = es*(|in| + |out| + |w|), a 1x1 stride-2 conv only
                         needs (and is only charged) every other row and column of its input.
                         A data gradient that also takes the backward sums of the BN layer below reads
                         that layer's input (es*|dx| more), and, when it closes a block, the other
                         gradient branch (es*|dx|) and the recorded ReLU bits of the layer below
                         (|dx|/8 bytes; as many again for an identity shortcut, whose gradient is the
                         block output's gradient under the block's own recorded bits)
  conv_wgrad             2*M*N*K flop;  bytes = es*(|x| + |dy|) + 4*|dw|
  bn_apply               2*es bytes/element (read x, write y) + es for the residual read (mode 2)
  bn_bwd_reduce          2*es bytes/element (read dz, x); launched only for the layers whose sums are not
                         taken in the output stage of the data gradient that produces dz (the stem, the
                         last block's residual-add layer and the projection shortcuts)
  bn_bwd_apply           3*es bytes/element (read dz, x, write dx) + 1/8 byte where the ReLU decision is
                         read from recorded bits (the residual-add layers and the projection shortcuts'
                         BN, whose incoming gradient is masked by the block's bits); no masked copy of the
                         shortcut's gradient is written
  lars_norms             8 bytes/parameter (read w, g)
  lars_apply             20 bytes/parameter (read w, g, v; write w, v) + 2 for the bf16 copy
The forward BN statistics and the other backward sums are part of conv_fwd / conv_dgrad (no bytes of
their own: they are taken from the output tile before it leaves the workgroup).
Peaks (MI355X, published): HBM 8 TB/s; dense bf16 MFMA 2.5 PFLOP/s; fp32 MFMA 157.3 TFLOP/s.
"""
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
MFMA_F32_PEAK_TFLOPS = 157.3

# HBM bytes per launch (fetch + write) from the rocprofv3 FETCH_SIZE / WRITE_SIZE counter runs summarized in
# profiles/resnet50_step_batch40_bf16_hbm_traffic.txt (batch 40, bf16), already scaled by the calibration
# copy; None where not measured.  Counter attribution per kernel is approximate: lines a kernel leaves
# dirty in L2 are written back during later kernels.  conv_wgrad includes its reduction pass.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {
    "conv_fwd": 39.93e6, "conv_dgrad": 63.54e6, "conv_wgrad": 62.64e6, "bn_apply": 42.55e6,
    "bn_bwd_reduce": 75.69e6, "bn_bwd_apply": 51.85e6, "lars_update": 383.55e6,
}

# Kernel classes of the step: (class, launch tags whose durations it sums, tag whose launches it is counted in).
# bn_finalize / bn_bwd_finalize (the passes from per-tile sums to per-channel statistics) and "other" (stem
# padding, weight transposition, pooling, classifier, cross-entropy) move next to nothing: they are listed with
# their time and no bound, so that the classes add up to all of the step's tagged kernel time.
CLASSES = [
    ("conv_fwd", ("conv_fwd",)), ("conv_dgrad", ("conv_dgrad",)), ("conv_wgrad", ("conv_wgrad", "splitk_reduce", "stem_unpad")),
    ("bn_apply", ("bn_apply",)), ("bn_bwd_reduce", ("bn_bwd_reduce",)), ("bn_bwd_apply", ("bn_bwd_apply",)),
    ("lars_update", ("lars_norms", "lars_apply")),
    ("bn_finalize", ("bn_finalize",)), ("bn_bwd_finalize", ("bn_bwd_finalize",)),
]


def layers(plan):
    """Conv+BN units of the plan in parameter order: dict(N,H,W,Cin,Cout,R,stride,P,mode)."""
    cfg = plan.cfg
    N = cfg.N
    out = []
    H = cfg.image_hw
    P = (H + 6 - 7) // 2 + 1
    out.append(dict(N=N, H=H, Cin=3, Cout=cfg.stem, R=7, stride=2, P=P, mode=1))
    H = (P - 1) // 2 + 1
    cin = cfg.stem
    for st in range(4):
        for b in range(cfg.blocks[st]):
            wd = cfg.widths[st]
            cout = wd * cfg.expansion
            stride = 2 if (b == 0 and st > 0) else 1
            Ho = (H + 2 - 3) // stride + 1
            out.append(dict(N=N, H=H, Cin=cin, Cout=wd, R=1, stride=1, P=H, mode=1))
            out.append(dict(N=N, H=H, Cin=wd, Cout=wd, R=3, stride=stride, P=Ho, mode=1))
            out.append(dict(N=N, H=Ho, Cin=wd, Cout=cout, R=1, stride=1, P=Ho, mode=2))
            if b == 0:
                out.append(dict(N=N, H=H, Cin=cin, Cout=cout, R=1, stride=stride, P=Ho, mode=0))
            H, cin = Ho, cout
    return out


def per_launch_cost(tag, plan):
    """List of (flops, bytes) per launch of `tag` within one step, in launch order."""
    es = 2 if plan.dtype == 1 else 4
    L = layers(plan)
    res = []

    def conv_cost(l, wgrad=False):
        m = l["N"] * l["P"] * l["P"]
        k = l["R"] * l["R"] * l["Cin"]
        flops = 2.0 * m * l["Cout"] * k
        x = l["N"] * l["H"] * l["H"] * l["Cin"]
        if l["R"] == 1 and l["stride"] == 2:
            x /= 4
        y = m * l["Cout"]
        w = l["Cout"] * k
        by = es * (x + y) + (4 * w if wgrad else es * w)
        return flops, by

    def elems(l):
        return l["N"] * l["P"] * l["P"] * l["Cout"]

    if tag == "conv_fwd":
        return _fwd_order(L, [conv_cost(l) for l in L])
    if tag in ("conv_dgrad", "conv_dgrad_fused_reads"):
        # conv_dgrad: the convolution's own bytes.  conv_dgrad_fused_reads: what its output stage reads on top
        # of that for the batch-norm backward sums it takes (bytes a separate reduce pass would otherwise read).
        out = []
        blocks = _blocks(L)[1:]
        for bi in range(len(blocks) - 1, -1, -1):
            b = blocks[bi]
            for j, l in enumerate(b):
                f, by = conv_cost(l)
                dx = l["N"] * l["H"] * l["H"] * l["Cin"]
                extra = 0.0
                if j in (1, 2):            # conv2, conv3: sums of the BN+ReLU layer below (its input is read)
                    extra = es * dx
                elif j == 0 and bi > 0:    # conv1 closes the block: + the shortcut's gradient, the previous
                    extra = 2 * es * dx + dx / 8   # block's BN input and its ReLU bits
                    if len(b) == 3:        # identity shortcut: its gradient is read under the block's bits
                        extra += dx / 8
                out.append((f, by) if tag == "conv_dgrad" else (0.0, extra))
        return out
    if tag == "conv_wgrad":
        return [conv_cost(l, True) for l in _bwd_order(L)]
    per_elem = {"bn_apply": (2 * es, es), "bn_bwd_reduce": (2 * es, 0), "bn_bwd_apply": (3 * es, 0.125)}
    if tag in per_elem:
        base, extra = per_elem[tag]
        seq = _fwd_order(L, L) if tag == "bn_apply" else _bwd_order(L)
        if tag == "bn_bwd_reduce":  # every other layer gets its sums from the data gradient that produces its dz
            last_add = [l for l in L if l["mode"] == 2][-1]
            seq = [l for l in seq if l["mode"] == 0 or l["Cin"] == 3 or l is last_add]
        bits = (2, 0) if tag == "bn_bwd_apply" else (2,)   # layers that read recorded ReLU bits / a residual
        return [(0.0, elems(l) * (base + (extra if l["mode"] in bits else 0))) for l in seq]
    # two launches each: every tensor but the stem's weight, then the stem's weight (whose gradient comes last)
    n_params, n_stem = sum(plan.sizes), plan.sizes[0]
    if tag == "lars_norms":
        return [(0.0, 8.0 * (n_params - n_stem)), (0.0, 8.0 * n_stem)]
    if tag == "lars_apply":
        per = 20.0 + (2.0 if plan.dtype == 1 else 0.0)
        return [(0.0, per * (n_params - n_stem)), (0.0, per * n_stem)]
    if tag == "lars_update":  # the whole update against the single-pass figure: w, g, v read, w, v written (+ bf16 copy)
        per = 20.0 + (2.0 if plan.dtype == 1 else 0.0)
        return [(0.0, per * (n_params - n_stem)), (0.0, per * n_stem)]
    raise KeyError(tag)


def _blocks(L):
    """Group layer records: [stem], then per block [c1, c2, c3, (proj)]."""
    out, i = [[L[0]]], 1
    while i < len(L):
        n = 4 if (i + 3 < len(L) and L[i + 3]["mode"] == 0) else 3
        out.append(L[i:i + n])
        i += n
    return out


def _fwd_order(L, vals):
    """The step launches c1, c2, proj, c3 per block."""
    idx = {id(l): v for l, v in zip(L, vals)}
    seq = []
    for b in _blocks(L):
        order = b if len(b) < 4 else [b[0], b[1], b[3], b[2]]
        seq += [idx[id(l)] for l in order]
    return seq


def _bwd_order(L):
    """Backward launches, per block from the last: c3, c2, c1, proj; the stem last."""
    seq = []
    bl = _blocks(L)
    for b in reversed(bl[1:]):
        seq += [b[2], b[1], b[0]] + ([b[3]] if len(b) == 4 else [])
    seq += bl[0]
    return seq


def class_record(name, tags, plan, tagged_ms, steps):
    """One kernel class: time per step summed over its tags' launches in `steps` sampled steps, against its bound."""
    ms = [t for tag, t in tagged_ms if tag in tags]
    rec = {"class": name, "tags": list(tags), "launches_per_step": len(ms) / steps, "time_per_step_ms": sum(ms) / steps}
    try:
        cost = per_launch_cost(name, plan)
    except KeyError:
        rec.update(bound=None, note="no algorithmic traffic of its own")
        return rec
    flops, nbytes = sum(c[0] for c in cost), sum(c[1] for c in cost)   # per step
    n = len(cost)
    main = [t for tag, t in tagged_ms if tag == tags[0]]
    if not ms or len(main) != n * steps:
        rec.update(bound=None, note=f"{len(main)} records of {tags[0]}, expected {n * steps}")
        return rec
    t = rec["time_per_step_ms"] * 1e-3
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if plan.dtype == 1 else MFMA_F32_PEAK_TFLOPS
    t_flop, t_byte = flops / (mfma_peak * 1e12), nbytes / (HBM_PEAK_GBS * 1e9)
    rec["launches_per_step"] = n
    rec["avg_launch_us"] = t * 1e6 / n
    if t_flop > t_byte:
        a = flops / t / 1e12
        rec.update(bound="mfma", achieved=a, peak=mfma_peak, unit="TFLOP/s", frac=a / mfma_peak)
    else:
        a = nbytes / t / 1e9
        rec.update(bound="hbm", achieved=a, peak=HBM_PEAK_GBS, unit="GB/s", frac=a / HBM_PEAK_GBS)
    rec["algorithmic_bytes_per_launch"] = nbytes / n
    rec["algorithmic_flops_per_launch"] = flops / n
    if name == "conv_dgrad":   # credited separately: the reads its output stage makes for the fused BN sums
        extra = sum(c[1] for c in per_launch_cost("conv_dgrad_fused_reads", plan))
        rec["fused_bn_read_bytes_per_launch"] = extra / n
        rec["frac_with_fused_reads"] = (nbytes + extra) / t / 1e9 / HBM_PEAK_GBS if rec["bound"] == "hbm" else None
    rec["traffic"] = MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(name) if (plan.dtype == 1 and plan.cfg.N == 40) else None
    return rec


def roofline(plan, tagged_ms, steps):
    """The bench line's roofline object from (tag, ms) records of every tagged launch in `steps` sampled steps:
    the class with the largest time per step (chosen from these measurements), with every class listed."""
    classes = [class_record(name, tags, plan, tagged_ms, steps) for name, tags in CLASSES]
    known = {t for _, tags in CLASSES for t in tags}
    other = [t for tag, t in tagged_ms if tag not in known]
    classes.append({"class": "other", "tags": sorted({tag for tag, _ in tagged_ms if tag not in known}),
                    "launches_per_step": len(other) / steps, "time_per_step_ms": sum(other) / steps, "bound": None})
    bounded = [c for c in classes if c.get("bound")]
    if not bounded:
        return {"kernel": None, "bound": None, "classes": classes}
    dom = max(bounded, key=lambda c: c["time_per_step_ms"])
    rec = {"kernel": dom["class"]}
    rec.update({k: v for k, v in dom.items() if k not in ("class",)})
    rec["chosen_by"] = "largest kernel time per step among the classes, from this run's own timings"
    rec["timing"] = ("dispatch begin/end timestamps of every tagged launch (events handed to hipExtLaunchKernel) in "
                     f"{steps} of the timed steps; kernels of the step's three streams overlap, so class times add up "
                     "to more than the step; a step whose launches all carry event packets is about twice as long as a "
                     "plain one, so its kernels overlap less than in the steps that make up ms_per_step")
    rec["kernel_time_per_step_ms"] = sum(c["time_per_step_ms"] for c in classes)
    rec["classes"] = classes
    return rec


def main():
    """python -m paper_1903_12650_amd.roofline <file with bench.py's JSON line> ...   prints the class table of each."""
    import json
    import sys
    print("%-26s %-16s %8s %8s %9s %6s %14s %8s %12s %8s" % ("workload", "class", "launches", "avg us", "ms/step", "bound",
                                                             "achieved", "of peak", "traffic MB", "x alg."))
    for path in sys.argv[1:]:
        line = [l for l in open(path).read().splitlines() if l.startswith("{")][-1]
        r = json.loads(line)
        wl = "step, batch %d, %s" % (r["config"]["global_batch"], r["dtype"])
        for c in r["roofline"]["classes"]:
            if c.get("bound"):
                tr = c.get("traffic")
                print("%-26s %-16s %8d %8.1f %9.3f %6s %9.0f %-4s %7.1f%% %12s %8s"
                      % (wl, c["class"], c["launches_per_step"], c["avg_launch_us"], c["time_per_step_ms"], c["bound"],
                         c["achieved"], c["unit"], 100 * c["frac"], "%.1f" % (tr / 1e6) if tr else "-",
                         "%.2f" % (tr / c["algorithmic_bytes_per_launch"]) if tr else "-"))
            else:
                print("%-26s %-16s %8d %8s %9.3f" % (wl, c["class"], c["launches_per_step"], "", c["time_per_step_ms"]))
        print("%-26s %-16s %8s %8s %9.3f   (step: %.3f ms; streams overlap)"
              % (wl, "all classes", "", "", r["roofline"]["kernel_time_per_step_ms"], r["ms_per_step"]))


if __name__ == "__main__":
    main()
