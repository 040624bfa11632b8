"""Per-shape timing of the convolution entry points on the 23 distinct convolution shapes of ResNet-50
v1.5 (forward, data gradient, weight gradient), each against its own roofline.

  python -m paper_1903_12650_amd.layer_bench [--batch 40] [--dtype bf16|f32] [--iters 6] [--passes fwd,dgrad,wgrad]
                                             [--cold] [--only "<shape>,<shape>"]

For every shape: the bound max(flops / MFMA peak, algorithmic bytes / HBM peak) in microseconds, then per
pass the launch duration (the library's dispatch timestamps) and bound / duration.  By default the buffers are
reused from iteration to iteration (warm caches: at batch 40 most operands stay in the 256 MB last-level cache);
with --cold every iteration works on its own copy of the tensors, enough copies that a pass has written and read
more than 512 MB before a copy comes round again, so every operand comes from HBM: the figure to hold against
the HBM bound.  Bytes are the minimum traffic of the pass (x, y, w once; a 1x1 stride-2 convolution is only
charged the quarter of x it needs); the weight gradient is timed with its split-K reduction.  Needs a GPU
and the built library; reads nothing but its arguments.
"""
import argparse

# (Cin, Cout, R, stride, Hin, occurrences in the network)
SHAPES = [(3, 64, 7, 2, 224, 1), (64, 64, 1, 1, 56, 1), (64, 64, 3, 1, 56, 3), (64, 256, 1, 1, 56, 4),
          (256, 64, 1, 1, 56, 2), (256, 128, 1, 1, 56, 1), (128, 128, 3, 2, 56, 1), (128, 512, 1, 1, 28, 4),
          (256, 512, 1, 2, 56, 1), (512, 128, 1, 1, 28, 3), (128, 128, 3, 1, 28, 3), (512, 256, 1, 1, 28, 1),
          (256, 256, 3, 2, 28, 1), (256, 1024, 1, 1, 14, 6), (512, 1024, 1, 2, 28, 1), (1024, 256, 1, 1, 14, 5),
          (256, 256, 3, 1, 14, 5), (1024, 512, 1, 1, 14, 1), (512, 512, 3, 2, 14, 1), (512, 2048, 1, 1, 7, 3),
          (1024, 2048, 1, 2, 14, 1), (2048, 512, 1, 1, 7, 2), (512, 512, 3, 1, 7, 2)]
HBM_PEAK, MFMA_BF16_PEAK, MFMA_F32_PEAK = 8.0e12, 2.5e15, 157.3e12


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=40)
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--iters", type=int, default=6)
    ap.add_argument("--passes", default="fwd,dgrad,wgrad")
    ap.add_argument("--cold", action="store_true")
    ap.add_argument("--only", default=None,
                    help="comma-separated shape labels to run, e.g. '128->128 3x3/1 @28,256->256 3x3/1 @14' (default: all)")
    args = ap.parse_args()
    passes = set(args.passes.split(","))
    import torch
    import paper_1903_12650_amd as rn

    bf = args.dtype == "bf16"
    tdt = torch.bfloat16 if bf else torch.float32
    es = 2 if bf else 4
    peak = MFMA_BF16_PEAK if bf else MFMA_F32_PEAK
    N = args.batch

    def timed(tags, f, copies):
        """Sum of the durations (us) of the launches with these tags in one call of f(copy index)."""
        for i in range(2):
            f(i % copies)
        torch.cuda.synchronize()
        total = 0.0
        for tag in tags:
            rn.profile_begin(tag, 64 * args.iters)
            for i in range(args.iters):
                f((i + 2) % copies)
            torch.cuda.synchronize()
            total += sum(rn.profile_end()) / args.iters * 1e3
        return total

    print("batch %d, %s, %s; microseconds; %% = roofline bound / measured"
          % (N, args.dtype, "cold (rotating tensor copies, > 512 MB between reuses)" if args.cold else "warm caches"))
    print("%-26s %3s %9s | %8s %5s | %8s %5s | %8s %5s" % ("shape", "x", "bound", "fwd", "%", "dgrad", "%", "wgrad", "%"))
    tot = dict(bound=0.0, fwd=0.0, dgrad=0.0, wgrad=0.0, flops=0.0)
    only = [o.strip() for o in args.only.split(",")] if args.only else None
    for (C, K, R, st, H, cnt) in SHAPES:
        if only is not None and ("%d->%d %dx%d/%d @%d" % (C, K, R, R, st, H)) not in only:
            continue
        pad = R // 2
        P = (H + 2 * pad - R) // st + 1
        per_copy = es * (N * H * H * C + N * P * P * K + K * R * R * C)
        copies = max(2, -(-(512 << 20) // per_copy)) if args.cold else 1
        copies = min(copies, args.iters + 2)
        xs = [torch.randn(N, H, H, C, device="cuda").to(tdt) for _ in range(copies)]
        ws_ = [(torch.randn(K, R, R, C, device="cuda") * 0.05).to(tdt) for _ in range(copies)]
        dys = [torch.randn(N, P, P, K, device="cuda").to(tdt) for _ in range(copies)]
        ys = [torch.empty_like(t) for t in dys]
        dxs = [torch.empty_like(t) for t in xs]
        dws = [torch.empty(K, R, R, C, device="cuda") for _ in range(copies)]
        x, w, dy = xs[0], ws_[0], dys[0]
        d = rn.ConvDesc(N, H, H, C, K, R, R, st, pad, rn.BF16 if bf else rn.F32)
        need = max(rn.conv_fwd_workspace_bytes(d), rn.conv_dgrad_workspace_bytes(d) if C != 3 else 0,
                   rn.conv_wgrad_workspace_bytes(d), 256)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        flops = 2.0 * N * P * P * K * R * R * C
        x_bytes = x.numel() / (4 if (R == 1 and st == 2) else 1)
        bound = max(flops / peak, es * (x_bytes + dy.numel() + w.numel()) / HBM_PEAK) * 1e6
        t_f = t_d = t_w = 0.0
        if "fwd" in passes:
            t_f = timed(["conv_fwd"], lambda i: rn.conv_fwd(xs[i], ws_[i], st, pad, y=ys[i], workspace=ws), copies)
        if "dgrad" in passes and C != 3:
            t_d = timed(["conv_dgrad"], lambda i: rn.conv_dgrad(dys[i], ws_[i], x.shape, st, pad, dx=dxs[i], workspace=ws),
                        copies)
        if "wgrad" in passes:
            t_w = timed(["conv_wgrad", "splitk_reduce"],
                        lambda i: rn.conv_wgrad(xs[i], dys[i], w.shape, st, pad, dw=dws[i], workspace=ws), copies)
        pct = lambda t: 100.0 * bound / t if t else 0.0
        print("%4d->%4d %dx%d/%d @%3d      x%d %9.1f | %8.1f %4.0f%% | %8.1f %4.0f%% | %8.1f %4.0f%%"
              % (C, K, R, R, st, H, cnt, bound, t_f, pct(t_f), t_d, pct(t_d), t_w, pct(t_w)))
        tot["bound"] += bound * cnt; tot["fwd"] += t_f * cnt; tot["dgrad"] += t_d * cnt; tot["wgrad"] += t_w * cnt
        tot["flops"] += flops * cnt
    print("whole network, one pass each: bound %.0f us; forward %.0f us (%.0f TFLOP/s), data gradient %.0f us, "
          "weight gradient %.0f us" % (tot["bound"], tot["fwd"], tot["flops"] / max(tot["fwd"], 1e-9) / 1e6, tot["dgrad"],
                                       tot["wgrad"]))


if __name__ == "__main__":
    main()
