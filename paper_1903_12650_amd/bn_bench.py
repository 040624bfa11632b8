"""Stand-alone timing of the batch-norm passes on the BN layer shapes of ResNet-50, each against the HBM roofline.

  python -m paper_1903_12650_amd.bn_bench [--batch 40] [--iters 8]

For every shape (spatial size, channels, with or without the residual add): the statistics pass, the forward apply
pass, the backward reduce pass and the backward apply pass of the stand-alone entry points (bn_relu_fwd,
bn_relu_bwd), timed by the library's dispatch timestamps on tensors rotated through enough copies that a pass has
moved more than 1 GB before a copy comes round again (nothing is cached), with the bytes each pass has to move
(2 B per element and operand in bf16) and the rate that gives.  Inside the training step the statistics and most
reduce passes do not exist (the convolutions' output stages take the sums); what remains are the apply passes, which
run next to other kernels there.  Needs a GPU and the built library; reads nothing but its arguments.
"""
import argparse

SHAPES = [(112, 64, 1), (56, 256, 2), (56, 64, 1), (28, 512, 2), (28, 128, 1), (14, 1024, 2), (14, 256, 1),
          (7, 2048, 2), (7, 512, 1)]  # (H = W, channels, BN mode: 1 = BN+ReLU, 2 = BN + residual + ReLU)
HBM_PEAK = 8.0e12


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=40)
    ap.add_argument("--iters", type=int, default=8)
    args = ap.parse_args()
    import torch
    import paper_1903_12650_amd as rn

    N = args.batch
    print("batch %d, bf16, uncached tensors; microseconds, TB/s, %% of the 8 TB/s HBM peak" % N)
    print("%-22s | %-22s | %-22s | %-22s | %-22s" % ("shape", "statistics (1 read)", "forward apply", "backward reduce (2 reads)",
                                                    "backward apply"))
    for (H, C, mode) in SHAPES:
        el = N * H * H * C
        copies = max(2, min(args.iters + 2, -(-(1 << 30) // (el * 2 * 3))))
        xs = [torch.randn(N, H, H, C, device="cuda").bfloat16() for _ in range(copies)]
        dzs = [torch.randn(N, H, H, C, device="cuda").bfloat16() for _ in range(copies)]
        rs = [torch.randn(N, H, H, C, device="cuda").bfloat16() for _ in range(copies)] if mode == 2 else [None] * copies
        g = torch.ones(C, device="cuda")
        b = torch.zeros(C, device="cuda")
        _, mean, rstd = rn.bn_relu_fwd(xs[0], g, b, rs[0], 1e-5, mode)
        masks = [rn.relu_mask_like(xs[0]).fill_(0x5a) for _ in range(copies)] if mode == 2 else [None] * copies

        def fwd(i):
            rn.bn_relu_fwd(xs[i], g, b, rs[i], 1e-5, mode)

        def bwd(i):
            rn.bn_relu_bwd(dzs[i], xs[i], None, g, mean, rstd, mode, beta=b, relu_mask=masks[i])

        def timed(tag, f):
            for i in range(2):
                f(i % copies)
            torch.cuda.synchronize()
            rn.profile_begin(tag, 64 * args.iters)
            for i in range(args.iters):
                f((i + 2) % copies)
            torch.cuda.synchronize()
            ms = rn.profile_end()
            return sum(ms) / len(ms) * 1e3

        cells = []
        # bytes per element: statistics read x; apply read x (+ residual), write z; reduce read dz, x; backward apply
        # read dz, x, write dx (+ dresidual for the residual-add layers of the stand-alone call)
        for tag, f, ops in (("bn_stats", fwd, 1), ("bn_apply", fwd, 3 if mode == 2 else 2), ("bn_bwd_reduce", bwd, 2),
                            ("bn_bwd_apply", bwd, 4 if mode == 2 else 3)):
            us = timed(tag, f)
            rate = el * 2 * ops / (us * 1e-6)
            cells.append("%6.1f us %4.1f TB/s %3.0f%%" % (us, rate / 1e12, 100 * rate / HBM_PEAK))
        print("%-22s | %s" % ("%dx%d C=%d mode %d" % (H, H, C, mode), " | ".join(cells)))


if __name__ == "__main__":
    main()
