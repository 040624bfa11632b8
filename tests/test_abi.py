"""The C-ABI library builds, loads, and exports every symbol that include/rn50_hip.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "rn50_hip.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", src)
    return sorted({n for n in names if n not in ("defined",) and not n.startswith("__")})


def test_library_exports_every_declared_symbol():
    lib_path = os.path.join(ROOT, "paper_1903_12650_amd", "librn50_hip.so")
    if not os.path.exists(lib_path):
        import importlib.util
        spec = importlib.util.spec_from_file_location("rn50_hip_build", os.path.join(ROOT, "paper_1903_12650_amd", "build.py"))
        build = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(build)
        build.build()
    lib = ctypes.CDLL(lib_path)
    names = _declared()
    assert len(names) >= 30, names
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in rn50_hip.h but not exported"
    for must in ("resnet_step", "conv_fwd", "conv_dgrad", "conv_wgrad", "bn_relu_fwd", "bn_relu_bwd", "xent_fwd_bwd",
                 "lars_update"):
        assert must in names


def test_host_side_argument_checks_need_no_gpu():
    import paper_1903_12650_amd as rn
    raw = rn.raw
    assert raw.rn50_version() >= 1
    # null descriptor / pointers are rejected before anything touches the device
    assert raw.conv_fwd(None, None, None, None, None, ctypes.c_size_t(0), None) == -1
    assert b"null" in raw.rn50_last_error()
    d = rn.ConvDesc(1, 8, 8, 12, 8, 3, 3, 1, 1, rn.BF16)
    one = ctypes.c_void_p(16)
    assert raw.conv_fwd(ctypes.byref(d), one, one, one, None, ctypes.c_size_t(0), None) == -2     # Cin % 8
    d = rn.ConvDesc(1, 8, 8, 16, 8, 3, 3, 1, 1, rn.BF16)
    assert raw.conv_fwd(ctypes.byref(d), ctypes.c_void_p(8), one, one, None, ctypes.c_size_t(0), None) == -4
    assert raw.conv_dgrad(ctypes.byref(d), one, one, one, one, ctypes.c_size_t(16), None) == -3
    assert rn.conv_dgrad_workspace_bytes(d) >= 8 * 9 * 16 * 2
    b = rn.BnDesc(2, 4, 4, 16, 1e-5, rn.BF16, 2)
    assert raw.bn_relu_fwd(ctypes.byref(b), one, one, one, None, one, None, one, one, None, None, ctypes.c_float(0.9), one,
                           ctypes.c_size_t(1 << 20), None) == -1                                # mode 2 without residual
    assert raw.xent_fwd_bwd(0, 10, one, one, ctypes.c_float(0), ctypes.c_float(1), one, one, one, None) == -1
    # the pooling kernels and the stem's padding kernel launch one grid plane per image and per row
    assert raw.maxpool_fwd(70000, 4, 4, 8, rn.BF16, one, one, None, None) == -2
    assert b"launch grid" in raw.rn50_last_error()
    assert raw.maxpool_bwd(70000, 4, 4, 8, rn.BF16, one, None, one, None, one, None) == -2
    stem = rn.ConvDesc(70000, 8, 8, 3, 64, 7, 7, 2, 3, rn.BF16)
    assert raw.conv_fwd(ctypes.byref(stem), one, one, one, one, ctypes.c_size_t(1 << 40), None) == -2


def test_dgrad_bn_sums_rejects_a_mask_without_addend_before_any_launch():
    """Every argument check of conv_dgrad_bn_sums precedes its first launch (the weight transposition): with no
    GPU here a launch attempt would surface as a HIP error (-5), an argument error comes back as -1."""
    import paper_1903_12650_amd as rn
    raw = rn.raw
    d = rn.ConvDesc(1, 8, 8, 16, 16, 3, 3, 1, 1, rn.BF16)
    one = ctypes.c_void_p(256)
    big = ctypes.c_size_t(1 << 30)
    rc = raw.conv_dgrad_bn_sums(ctypes.byref(d), one, one, one, None, one, one, None, one, one, one, one, one, big, one,
                                big, None)
    assert rc == -1 and b"addend_mask without addend" in raw.rn50_last_error()


def test_plan_creation_checks_shapes_and_frees_the_plan_on_error():
    import paper_1903_12650_amd as rn
    with __import__("pytest").raises(rn.Rn50Error) as e:
        rn.ResnetPlan(8, rn.BF16, 64, 70000, (8, 8, 8, 8), (1, 1, 1, 1), 8, 4)     # more classes than xent covers
    assert e.value.code == -2
    with __import__("pytest").raises(rn.Rn50Error) as e:
        rn.ResnetPlan(8, rn.BF16, 64, 10, (8, 8, 8, 12), (1, 1, 1, 1), 8, 4)       # width not a multiple of 8
    assert e.value.code == -2
    assert rn.raw.resnet_plan_prepare(None) == -1


def test_loop_entry_points_check_their_arguments_without_a_gpu():
    import paper_1903_12650_amd as rn
    raw = rn.raw
    plan = rn.ResnetPlan(8, rn.BF16, 64, 10, (8, 8, 8, 8), (1, 1, 1, 1), 8, 4)
    one = ctypes.c_void_p(256)
    sched = rn.LrSchedule(1.0)
    f = ctypes.c_float
    assert raw.resnet_train_step(plan.handle, None, one, f(0.9), one, one, one, one, one, one, one, None, one,
                                 ctypes.c_size_t(1 << 40), None) == -1                      # no schedule
    assert raw.resnet_train_step(plan.handle, ctypes.byref(rn.LrSchedule(1.0, decay="step", step_every=0)), one, f(0.9), one,
                                 one, one, one, one, one, one, None, one, ctypes.c_size_t(1 << 40), None) == -1
    assert b"step_every" in raw.rn50_last_error()
    assert raw.resnet_train_step(plan.handle, ctypes.byref(sched), ctypes.c_void_p(8), f(0.9), one, one, one, one, one, one,
                                 one, None, one, ctypes.c_size_t(1 << 40), None) == -4            # misaligned state
    assert raw.resnet_train_step(plan.handle, ctypes.byref(sched), one, f(0.9), one, one, one, one, one, one, one, None,
                                 one, ctypes.c_size_t(16), None) == -3                             # workspace too small
    assert raw.resnet_train_state_init(plan.handle, one, ctypes.c_size_t(8), ctypes.c_int64(0), None) == -3
    assert raw.resnet_train_state_init(plan.handle, one, ctypes.c_size_t(1 << 30), ctypes.c_int64(-1), None) == -1
    assert raw.resnet_init_params(plan.handle, ctypes.c_uint64(1), None, None, None, None) == -1
    assert raw.resnet_eval(plan.handle, one, one, None, one, one, None, one, one, one, ctypes.c_size_t(1 << 40), None) == -1
    assert raw.top1_accuracy(0, 10, one, one, one, one, None) == -1
    b = rn.BnDesc(2, 4, 4, 16, 1e-5, rn.BF16, 2)
    assert raw.bn_relu_infer(ctypes.byref(b), one, one, one, one, one, None, one, one, ctypes.c_size_t(256), None) == -1
    n_bn = raw.resnet_plan_num_bn(plan.handle)
    assert n_bn == 1 + 3 * 4 + 4 and int(raw.resnet_plan_bn_channels(plan.handle)) % 64 == 0
    c = ctypes.c_int()
    assert int(raw.resnet_plan_bn_offset(plan.handle, 0, ctypes.byref(c))) == 0 and c.value == 8
    assert int(raw.resnet_plan_bn_offset(plan.handle, n_bn, None)) == -1
    assert int(raw.resnet_train_state_bytes(plan.handle)) == 256 + 8 * int(raw.resnet_plan_bn_channels(plan.handle))


def test_plan_matches_the_oracles_parameter_table():
    import paper_1903_12650_amd as rn
    from oracle import net
    plan = rn.ResnetPlan(40, rn.BF16)
    table = net.param_table()
    assert plan.num_tensors == 161 and sum(plan.sizes) == 25_557_032
    for (name, shape, _), ps in zip(table, plan.shapes):
        assert tuple(shape) == tuple(ps), name
    assert all(o % 64 == 0 for o in plan.offsets)
    assert plan.workspace_bytes > 0 and plan.arena_elems >= sum(plan.sizes)


def test_roofline_cost_model_totals():
    """Algorithmic totals per step at batch 40 match the hand-derived figures: ~8.17 GFLOP/image of
    forward convolution, 444.6 M BN elements."""
    import paper_1903_12650_amd as rn
    from paper_1903_12650_amd import roofline as rl
    plan = rn.ResnetPlan(40, rn.BF16)
    fwd = rl.per_launch_cost("conv_fwd", plan)
    assert len(fwd) == 53 and len(rl.per_launch_cost("conv_dgrad", plan)) == 52
    gflop_per_image = sum(f for f, _ in fwd) / 40 / 1e9
    assert abs(gflop_per_image - 8.17) < 0.05, gflop_per_image
    apply = rl.per_launch_cost("bn_apply", plan)          # 2 tensors per element + the residual of the add layers
    assert len(apply) == 53
    red = rl.per_launch_cost("bn_bwd_reduce", plan)       # the stem, the last residual-add layer, 4 projections
    assert len(red) == 6
    bwd = rl.per_launch_cost("bn_bwd_apply", plan)        # 3 tensors per element + recorded bits where they are read
    L = rl.layers(plan)
    E = sum(l["N"] * l["P"] * l["P"] * l["Cout"] for l in L)
    E_add = sum(l["N"] * l["P"] * l["P"] * l["Cout"] for l in L if l["mode"] == 2)
    E_proj = sum(l["N"] * l["P"] * l["P"] * l["Cout"] for l in L if l["mode"] == 0)
    assert abs(E / 1e6 - 444.6) < 0.5
    assert sum(b for _, b in apply) == 4 * E + 2 * E_add and sum(b for _, b in bwd) == 6 * E + (E_add + E_proj) / 8
    assert sum(b for _, b in rl.per_launch_cost("lars_apply", plan)) == 22 * 25_557_032
