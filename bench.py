"""Benchmark: ResNet-50 v1.5 training step (forward, backward, LARS) on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch 40] [--dtype bf16|f32]

Prints ONE JSON line: images/s for whole training steps at batch 40 (one worker's share of the
paper's 81,920-image minibatch), with inputs, parameters and workspace resident in HBM before
the timed region, plus
  "roofline":     achieved vs peak for the step's dominant kernel class (the one with the largest kernel
                  time, chosen from this run's timings) and for every other class, from HIP events the
                  library hands to every tagged launch in a sample of the timed steps, and
  "cpu_baseline": the CPU oracle timed on a bounded sample of the same workload,
  "train_loop":   the same step inside the training loop (device-side learning-rate schedule and step
                  counter, BN moving averages, label smoothing), launched eagerly and as replays of one
                  captured HIP graph.
Synthetic data: N(0,1) images of ImageNet's shape, uniform labels, He-normal weights.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--batch", type=int, default=40)
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--no-train-loop", action="store_true")
    ap.add_argument("--fuse-conv3-input", action="store_true",
                    help="conv3 of every block applies conv2's BN+ReLU in its operand load (same results; for timing)")
    ap.add_argument("--sample-every", type=int, default=200,
                    help="per-launch timing in every n-th timed step (a step whose launches are all timed takes about twice "
                         "as long; it is part of the timed region, so with the defaults it costs the reported rate 0.6 %%)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of known size (the float master arena) before the steps: "
                         "the reference dispatch that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def build_state(rn, N, dtype):
    import numpy as np
    import torch
    import synth
    bf = dtype == "bf16"
    plan = rn.ResnetPlan(N, rn.BF16 if bf else rn.F32)
    table = [("t%d" % i, s, "conv" if len(s) == 4 else ("fcw" if len(s) == 2 else ("gamma" if i % 3 == 1 else "beta")))
             for i, s in enumerate(plan.shapes)]
    table[-1] = (table[-1][0], table[-1][1], "fcb")
    params = synth.params_from_table(synth.DEFAULT_SEED, table)
    M = torch.zeros(plan.arena_elems, dtype=torch.float32)
    for off, p in zip(plan.offsets, params):
        M[off:off + p.size] = torch.from_numpy(p.ravel())
    M = M.cuda()
    S = dict(plan=plan, M=M, V=torch.zeros_like(M), G=torch.zeros_like(M),
             Mod=M.to(torch.bfloat16) if bf else M,
             ws=torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda"),
             loss=torch.zeros(1, device="cuda"))
    img = synth.activation_nhwc(synth.DEFAULT_SEED, "img", N, 3, 224, 224)
    S["images"] = torch.from_numpy(img).cuda().to(torch.bfloat16 if bf else torch.float32)
    S["labels"] = torch.from_numpy(synth.labels(synth.DEFAULT_SEED, "lab", N, 1000)).cuda()
    return S


def cpu_one_thread():
    """The oracle on one thread for the three small configurations (one bottleneck block in float at batch 2,
    forward + backward; the LARS update over ResNet-50's 161 tensors; one convolution shape of the sweep, forward,
    at batch 4): seconds each."""
    import ctypes
    import numpy as np
    import oracle as orc
    import synth
    from oracle import net
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        before = gomp.omp_get_max_threads()
        gomp.omp_set_num_threads(1)
    except OSError:
        return {"note": "libgomp not found: no one-thread figure"}
    try:
        rec = {"threads": 1}
        x = synth.activation_nhwc(synth.DEFAULT_SEED, "x", 2, 64, 56, 56)
        ws = [synth.conv_weight_krsc(synth.DEFAULT_SEED, "w%d" % i, k, c, r, r)
              for i, (k, c, r) in enumerate(((64, 64, 1), (64, 64, 3), (256, 64, 1), (256, 64, 1)))]
        t0 = time.perf_counter()
        y1 = orc.conv_fwd(x, ws[0], 1, 0); y2 = orc.conv_fwd(y1, ws[1], 1, 1); y3 = orc.conv_fwd(y2, ws[2], 1, 0)
        ys = orc.conv_fwd(x, ws[3], 1, 0)
        for (a, w, yy, pad) in ((y2, ws[2], y3, 0), (y1, ws[1], y2, 1), (x, ws[0], y1, 0), (x, ws[3], ys, 0)):
            orc.conv_dgrad(yy, w, a.shape, 1, pad); orc.conv_wgrad(a, yy, w.shape, 1, pad)
        rec["config1_block_convs_fwd_bwd_batch2_s"] = time.perf_counter() - t0
        table = net.param_table()
        params = synth.params_from_table(synth.DEFAULT_SEED, table)
        grads = synth.grads_from_table(synth.DEFAULT_SEED, table, 1e-3)
        vel = [np.zeros_like(p) for p in params]
        t0 = time.perf_counter()
        orc.lars_update(params, grads, vel, 0.001, 0.9, 1.0, net.lars_hyper(table, 5e-5))
        rec["config2_lars_161_tensors_s"] = time.perf_counter() - t0
        x = synth.round_bf16(synth.activation_nhwc(synth.DEFAULT_SEED, "x3", 4, 256, 14, 14))
        w = synth.round_bf16(synth.conv_weight_krsc(synth.DEFAULT_SEED, "w3", 256, 256, 3, 3))
        t0 = time.perf_counter()
        orc.conv_fwd(x, w, 1, 1)
        rec["config3_conv3x3_256_14x14_fwd_batch4_s"] = time.perf_counter() - t0
        return rec
    finally:
        gomp.omp_set_num_threads(before)


def cpu_baseline(batch_sample=40):
    """The oracle's training step (forward, backward, LARS) on a bounded sample: `batch_sample`
    images of the same 224x224 workload, all host cores OpenMP gives it."""
    import numpy as np
    import oracle  # noqa: F401
    import synth
    from oracle import net
    table = net.param_table()
    master = synth.params_from_table(synth.DEFAULT_SEED, table)
    model = [synth.round_bf16(p) for p in master]
    vel = [np.zeros_like(p) for p in master]
    img = synth.round_bf16(synth.activation_nhwc(synth.DEFAULT_SEED, "img", batch_sample, 3, 224, 224))
    lab = synth.labels(synth.DEFAULT_SEED, "lab", batch_sample, 1000)
    t0 = time.perf_counter()
    net.train_step(img, lab, master, model, vel, table)
    dt = time.perf_counter() - t0
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    return {"value": batch_sample / dt, "unit": "images/s", "cores": cores, "kind": "oracle",
            "sample": f"one full training step (fwd+bwd+LARS) of ResNet-50 on {batch_sample} of the 40 images, "
                      f"{dt:.1f} s wall",
            "one_thread": cpu_one_thread()}


def train_loop_record(rn, torch, S, steps, warmup, batch):
    """ms/step of resnet_train_step (warm-up + polynomial decay on the device, moving averages on),
    eager and as replays of one captured graph."""
    plan = S["plan"]
    state = rn.TrainState(plan)
    sched = rn.LrSchedule(base_lr=1.0, warmup_steps=5, warmup_start_lr=0.1, decay="polynomial", total_steps=100000,
                          end_lr=1e-4, power=2.0)

    def step():
        rn.resnet_train_step(plan, sched, state, S["images"], S["labels"], S["M"], S["V"], S["G"], S["Mod"], S["ws"],
                             loss_out=S["loss"])

    def timed(f):
        for _ in range(warmup):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    rec = {"schedule": "linear warm-up 5 steps, polynomial (power 2) decay", "bn_momentum": 0.9}
    ms = timed(step)
    rec.update(ms_per_step_eager=ms, images_per_s_eager=batch / (ms * 1e-3))
    try:
        st = torch.cuda.Stream()
        st.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            step()
        torch.cuda.synchronize()
        ms = timed(g.replay)
        rec.update(ms_per_step_graph=ms, images_per_s_graph=batch / (ms * 1e-3))
    except Exception as e:  # the eager figure stands on its own
        rec["graph_error"] = str(e)[:200]
    rec["steps_taken"] = state.step
    rec["loss"] = float(S["loss"].item())
    return rec


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the batch-40 share of one worker); "
              "--gpus %d is not supported, no multi-GPU figure is produced" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_1903_12650_amd as rn
    from paper_1903_12650_amd import roofline as rl

    S = build_state(rn, args.batch, args.dtype)
    plan = S["plan"]
    if args.fuse_conv3_input:
        plan.fuse_conv3_input(True)

    def step():
        rn.resnet_step(plan, S["images"], S["labels"], S["M"], S["V"], S["G"], S["Mod"], 1.0, S["ws"], update=True,
                       loss_out=S["loss"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibration_copy:
        scratch = torch.empty_like(S["M"])
        scratch.copy_(S["M"])          # reads and writes 4 * arena_elems bytes
        torch.cuda.synchronize()
        print("calibration copy: %d bytes read, %d bytes written" % (4 * plan.arena_elems, 4 * plan.arena_elems),
              file=sys.stderr)
    sampling = not args.no_roofline
    if sampling:
        rn.profile_begin("", (args.steps // args.sample_every + 2) * 1024)   # every tagged launch of the sampled steps
        rn.profile_pause(True)
    # Every step is bracketed by a pair of events on the stream the step is launched on (its side streams
    # fork from and join back into it); the kernels' own durations are timed in every n-th step only.
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    sampled = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if sampling:
            rn.profile_pause(i % args.sample_every != 0)
            sampled += i % args.sample_every == 0
        ev[i][0].record()
        step()
        ev[i][1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt / args.steps * 1e3
    step_ms = sorted(a.elapsed_time(b) for a, b in ev)
    plain = sorted(a.elapsed_time(b) for i, (a, b) in enumerate(ev) if not sampling or i % args.sample_every != 0) or step_ms
    out = {"metric": f"ResNet-50 train images/sec on 1 MI355X, batch {args.batch} {args.dtype}",
           "value": args.batch / (ms * 1e-3),
           "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype,
           "data": "synthetic",
           "config": {"workload": f"full ResNet-50 v1.5 training step (fwd+bwd+LARS), batch {args.batch}, 224x224, "
                                  f"1000 classes, {args.dtype} activations with fp32 master weights",
                      "global_batch": args.batch, "loss": float(S["loss"].item())},
           "step_ms_events": {"median": step_ms[len(step_ms) // 2], "min": step_ms[0], "max": step_ms[-1],
                              "median_of_steps_without_launch_timing": plain[len(plain) // 2],
                              "steps_with_launch_timing": sampled,
                              "mean_of_steps_with_launch_timing": (sum(a.elapsed_time(b) for i, (a, b) in enumerate(ev)
                                                                       if i % args.sample_every == 0) / sampled
                                                                   if sampling and sampled else None),
                              "note": "hipEvent pairs around every timed step on the launch stream; the steps with "
                                      "launch timing are part of the timed region and of ms_per_step"}}
    if sampling:
        durations_ms = rn.profile_end()
        out["roofline"] = rl.roofline(plan, list(zip(rn.profile_tags(), durations_ms)), sampled)
        out["roofline"]["timed_steps"] = sampled
    if not args.no_train_loop:
        out["train_loop"] = train_loop_record(rn, torch, S, args.steps, args.warmup, args.batch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
