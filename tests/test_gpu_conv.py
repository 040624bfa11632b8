"""GPU parity: convolution forward / data gradient / weight gradient against the oracle."""
import numpy as np
import pytest
import torch

import oracle as orc
import synth
from gpu_util import TOL, assert_close, dev, host, inputs

pytestmark = pytest.mark.gpu
SEED = synth.DEFAULT_SEED


@pytest.fixture(scope="module")
def rn():
    import paper_1903_12650_amd as rn
    return rn


def run_case(rn, mode_name, N, H, W, C, K, R, stride, pad, do_dgrad=True, tag=""):
    bf = mode_name == "bf16"
    tol = TOL[mode_name]
    x = synth.activation_nhwc(SEED, "x" + tag, N, C, H, W)
    w = synth.conv_weight_krsc(SEED, "w" + tag, K, C, R, R)
    x, w = inputs(mode_name, x, w)
    y_o = orc.conv_fwd(x, w, stride, pad)
    dy = synth.activation_nhwc(SEED, "dy" + tag, N, K, y_o.shape[1], y_o.shape[2])
    dy, = inputs(mode_name, dy)
    xd, wd, dyd = dev(x, bf), dev(w, bf), dev(dy, bf)
    errs = {}
    y = rn.conv_fwd(xd, wd, stride, pad)
    errs["y"] = assert_close(y, y_o, tol, f"y {tag}")
    dw = rn.conv_wgrad(xd, dyd, w.shape, stride, pad)
    assert dw.dtype == torch.float32
    errs["dw"] = assert_close(dw, orc.conv_wgrad(x, dy, w.shape, stride, pad), tol, f"dw {tag}")
    if do_dgrad:
        dx = rn.conv_dgrad(dyd, wd, x.shape, stride, pad)
        errs["dx"] = assert_close(dx, orc.conv_dgrad(dy, w, x.shape, stride, pad), tol, f"dx {tag}")
    return errs


SMALL = [  # N,H,W,C,K,R,stride,pad : ragged tiles, tails, every stride/pad/filter combination
    (2, 9, 7, 8, 8, 1, 1, 0),
    (1, 12, 12, 16, 24, 3, 1, 1),
    (3, 11, 13, 24, 40, 3, 2, 1),
    (2, 10, 10, 72, 136, 1, 2, 0),
    (1, 17, 15, 136, 72, 3, 1, 1),
    (2, 8, 8, 64, 64, 3, 2, 1),
    (1, 5, 5, 8, 200, 3, 1, 0),
    (5, 14, 14, 256, 64, 1, 1, 0),
    (2, 14, 14, 64, 256, 1, 1, 0),
    (1, 20, 20, 8, 8, 7, 2, 3),
    (2, 6, 6, 16, 16, 5, 1, 2),
    (1, 1, 1, 8, 8, 1, 1, 0),
    (2, 9, 7, 16, 16, 1, 2, 0),      # stride 2, odd sizes: the four pixel parity classes differ in size
    (1, 1, 5, 8, 8, 3, 2, 1),        # a single row: two parity classes are empty
    (2, 5, 4, 8, 16, 2, 2, 0),       # even filter, stride 2
    # 3x3 stride 1 pad 1 with whole 128-byte channel chunks, several tiles and images per case
    (3, 9, 9, 64, 64, 3, 1, 1),      # tiles that span two images, short last tile
    (2, 5, 12, 128, 72, 3, 1, 1),    # two channel chunks, ragged column tile
    (5, 7, 21, 192, 64, 3, 1, 1),    # three channel chunks (odd number of pipeline steps)
    (7, 4, 48, 64, 128, 3, 1, 1),    # wide, low images
    (2, 1, 56, 64, 64, 3, 1, 1),     # one-row images: every tap row but the middle one is padding
    (3, 8, 8, 128, 128, 3, 1, 1),    # one 64-pixel tile per image
    (1, 1, 1, 8, 8, 3, 1, 1),        # a single pixel: eight of the nine taps are padding
    (2, 2, 2, 16, 8, 3, 1, 1),       # 2x2 images: every pixel is a corner
    (1, 3, 100, 8, 8, 3, 1, 1),      # too wide for the one-run kernels (run of 2W + 2 rows): the general path
    (2, 3, 62, 8, 16, 3, 1, 1),      # the widest image the nine-tap weight gradient takes
]


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
@pytest.mark.parametrize("case", SMALL)
def test_small_shapes(rn, mode_name, case):
    N, H, W, C, K, R, stride, pad = case
    if mode_name == "f32":
        C = max(4, C // 2); K = max(4, K // 2)          # float needs only multiples of 4
    run_case(rn, mode_name, N, H, W, C, K, R, stride, pad, tag=str(case))


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
@pytest.mark.parametrize("N,HW", [(2, 32), (1, 38), (3, 224)])
def test_stem(rn, mode_name, N, HW):
    """3-channel 7x7/2 pad-3 stem (appendix log: [3(4),224,224] -> (64,112,112))."""
    run_case(rn, mode_name, N, HW, HW, 3, 64, 7, 2, 3, do_dgrad=False, tag=f"stem{N}x{HW}")


# The 23 distinct convolution shapes of ResNet-50 v1.5: Cin, Cout, R, stride, Hin
RESNET_SHAPES = [
    (3, 64, 7, 2, 224), (64, 64, 1, 1, 56), (64, 64, 3, 1, 56), (64, 256, 1, 1, 56), (256, 64, 1, 1, 56),
    (256, 128, 1, 1, 56), (128, 128, 3, 2, 56), (128, 512, 1, 1, 28), (256, 512, 1, 2, 56), (512, 128, 1, 1, 28),
    (128, 128, 3, 1, 28), (512, 256, 1, 1, 28), (256, 256, 3, 2, 28), (256, 1024, 1, 1, 14), (512, 1024, 1, 2, 28),
    (1024, 256, 1, 1, 14), (256, 256, 3, 1, 14), (1024, 512, 1, 1, 14), (512, 512, 3, 2, 14), (512, 2048, 1, 1, 7),
    (1024, 2048, 1, 2, 14), (2048, 512, 1, 1, 7), (512, 512, 3, 1, 7),
]


@pytest.mark.parametrize("shape", RESNET_SHAPES)
def test_resnet50_shapes_batch40_bf16(rn, shape):
    """BASELINE config 3: every distinct conv shape at batch 40, bf16, fwd + dgrad + wgrad."""
    C, K, R, stride, H = shape
    errs = run_case(rn, "bf16", 40, H, H, C, K, R, stride, R // 2, do_dgrad=(C != 3), tag=str(shape))
    print(shape, {k: "%.2e" % v for k, v in errs.items()})


@pytest.mark.parametrize("shape", [(64, 64, 3, 1, 56), (256, 512, 1, 2, 56), (512, 512, 3, 2, 14), (3, 64, 7, 2, 224)])
def test_resnet50_shapes_f32(rn, shape):
    C, K, R, stride, H = shape
    run_case(rn, "f32", 4, H, H, C, K, R, stride, R // 2, do_dgrad=(C != 3), tag=str(shape))


def test_conv_reproducible_and_workspace_poison(rn):
    """Same inputs twice -> identical bits, with a NaN-poisoned workspace (nothing unwritten is read)."""
    x = dev(synth.activation_nhwc(SEED, "x", 8, 128, 28, 28), True)
    w = dev(synth.conv_weight_krsc(SEED, "w", 128, 128, 3, 3), True)
    dy = dev(synth.activation_nhwc(SEED, "dy", 8, 128, 14, 14), True)
    d = rn.ConvDesc(8, 28, 28, 128, 128, 3, 3, 2, 1, rn.BF16)
    outs = []
    for _ in range(2):
        ws = torch.full((max(rn.conv_wgrad_workspace_bytes(d), rn.conv_dgrad_workspace_bytes(d), 256) // 4,), float("nan"),
                        device="cuda").view(torch.uint8)
        outs.append((rn.conv_fwd(x, w, 2, 1), rn.conv_dgrad(dy, w, x.shape, 2, 1, workspace=ws.clone()),
                     rn.conv_wgrad(x, dy, w.shape, 2, 1, workspace=ws.clone())))
    for a, b in zip(*outs):
        assert torch.equal(a, b) and torch.isfinite(a.float()).all()


def test_conv_error_codes(rn):
    x = torch.zeros((1, 8, 8, 12), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((8, 3, 3, 12), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rn.Rn50Error) as e:
        rn.conv_fwd(x, w, 1, 1)                              # Cin = 12 is not a multiple of 8
    assert e.value.code == -2
    x = torch.zeros((1, 8, 8, 16), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((8, 3, 3, 16), dtype=torch.bfloat16, device="cuda")
    dy = torch.zeros((1, 8, 8, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rn.Rn50Error) as e:
        rn.conv_dgrad(dy, w, x.shape, 1, 1, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
    x3 = torch.zeros((1, 16, 16, 3), dtype=torch.bfloat16, device="cuda")
    w3 = torch.zeros((64, 7, 7, 3), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rn.Rn50Error) as e:
        rn.conv_dgrad(torch.zeros((1, 8, 8, 64), dtype=torch.bfloat16, device="cuda"), w3, x3.shape, 2, 3)
    assert e.value.code == -2


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
def test_3x3_taps_never_reach_into_the_neighbouring_image(rn, mode_name):
    """The 3x3 / stride 1 kernels read one contiguous run of pixels per tile, which spans image borders: with one
    image of the batch all NaN (forward: of x; data gradient: of dy), the other images' outputs are bit for bit
    those of the batch where that image is zero."""
    bf = mode_name == "bf16"
    N, H, W, C, K = 3, 6, 10, (64 if bf else 32), (64 if bf else 32)
    x, w, dy = inputs(mode_name, synth.activation_nhwc(SEED, "x", N, C, H, W), synth.conv_weight_krsc(SEED, "w", K, C, 3, 3),
                      synth.activation_nhwc(SEED, "dy", N, K, H, W))
    wd = dev(w, bf)
    outs = []
    for poison in (0.0, float("nan")):
        xd, dyd = dev(x, bf).clone(), dev(dy, bf).clone()
        xd[1] = poison
        dyd[1] = poison
        outs.append((rn.conv_fwd(xd, wd, 1, 1), rn.conv_dgrad(dyd, wd, xd.shape, 1, 1)))
    for a, b in zip(*outs):
        assert torch.equal(a[0], b[0]) and torch.equal(a[2], b[2])
        assert torch.isnan(b[1]).any()
