"""xnor_forward_image (few-channel images, whole forward pass in one kernel) against the oracle.

The expected values are the oracle's forward pass on the same fp32 tensors: binary dot products bit
for bit, the fp32 output within 1e-5 relative (one fp32 subnormal spacing where that is larger) and
zero exactly where the oracle is zero.  The shapes cover every template of the kernel (kernel size
3 / 5 / 7, one to four channels, one and several filters, strides), images narrower than a wave and wider
than several, heights below one band and across bands, padding from none to more than the kernel,
and the paper's own sizes (Tables I-III: one channel, one 3x3 filter, 256^2 ... 2048^2).
"""
import zlib

import numpy as np
import pytest
import torch

import oracle
from paper_2007_14178_amd.workloads import random_layer

pytestmark = pytest.mark.gpu
RTOL = 1e-5


@pytest.fixture(scope="module")
def xb():
    from paper_2007_14178_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def assert_out(got, ref, what, floor=2.0 ** -149):
    got = got.astype(np.float64); ref = ref.astype(np.float64)
    assert got.shape == ref.shape, what
    err = np.abs(got - ref)
    bad = err > np.maximum(RTOL * np.abs(ref), floor)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside {RTOL} rel; worst {err.max()}"
    assert np.array_equal(got == 0, ref == 0), f"{what}: zero pattern differs"


def run_case(xb, shape, tag=""):
    N, C, H, W, F, k, pad = shape[:7]
    sh, sw = shape[7:] if len(shape) > 7 else (1, 1)
    full = (N, C, H, W, F, k, k, sh, sw, pad, pad)
    rng = np.random.default_rng(zlib.crc32(("image" + tag + str(shape)).encode()))
    layer, I, Wt = random_layer(rng, "t", *full)
    s = xb.Shape(*full)
    assert xb.xnor_forward_image_supported(s)
    d_ref, K_ref, a_ref, O_ref = oracle.forward(I, Wt, oracle.Shape(*full))
    dI = dev(I)
    Wpk, alpha, _ = xb.xnor_filter_prepare(dev(Wt))
    out, dot = xb.xnor_forward_image(dI, Wpk, alpha, s, want_dot=True)
    torch.cuda.synchronize()
    assert np.array_equal(dot.cpu().numpy(), d_ref), "dot"
    # (in fp32's subnormal range: this kernel sums K in fp32, kw*C + kh roundings of half a spacing
    # each, times |dot| * alpha; K * alpha is rounded again, times |dot|, and so is the product)
    kr = k * C + k
    floor = (0.5 * np.abs(d_ref.astype(np.float64)) * (kr * a_ref.astype(np.float64)[None, :, None, None] + 1.0) + 1.0) * 2.0 ** -149
    assert_out(out.cpu().numpy(), O_ref, "out", floor)
    # without the optional dots the output is the same, bit for bit
    out2, none = xb.xnor_forward_image(dI, Wpk, alpha, s)
    torch.cuda.synchronize()
    assert none is None and torch.equal(out, out2)
    return s, dI, Wpk, alpha, out, dot


#   N  C   H    W   F  k  pad
SHAPES = [
    (1, 1, 5, 5, 1, 3, 1),
    (1, 1, 1, 1, 1, 3, 1),          # a single pixel: every tap but the centre is padding
    (2, 1, 2, 70, 1, 3, 1),         # image lower than the kernel
    (2, 1, 7, 70, 1, 3, 0),         # no padding, two column tiles, ragged
    (1, 1, 40, 63, 2, 3, 1),
    (1, 1, 33, 64, 1, 3, 2),
    (3, 1, 100, 65, 1, 3, 1),       # several bands per image
    (1, 2, 19, 130, 3, 3, 1),
    (2, 3, 37, 41, 5, 3, 1),        # a three-channel first layer
    (1, 4, 9, 200, 7, 3, 3),        # padding as wide as the kernel: windows that are all padding
    (1, 1, 30, 50, 1, 5, 2),
    (2, 2, 12, 77, 4, 5, 0),
    (1, 3, 23, 66, 6, 5, 4),        # window rows spread over three words
    (1, 4, 16, 35, 2, 5, 2),        # one window row per word
    (1, 1, 20, 90, 1, 7, 3),        # two words per window
    (2, 2, 15, 64, 3, 7, 3),
    (1, 3, 31, 47, 8, 7, 6),
    (1, 4, 10, 129, 2, 7, 1),
    (1, 1, 300, 300, 1, 3, 1),
    (1, 3, 224, 224, 16, 3, 1),     # an ImageNet-sized three-channel input
    (1, 1, 64, 64, 600, 3, 1),      # many filters
    # strides (sh, sw)
    (1, 3, 224, 224, 8, 7, 3, 2, 2),    # a ResNet-style first layer
    (2, 1, 50, 131, 2, 3, 1, 2, 1),
    (1, 2, 41, 70, 3, 5, 0, 1, 3),
    (1, 4, 33, 65, 2, 3, 1, 3, 2),
    (1, 1, 9, 9, 1, 7, 3, 4, 4),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_image_forward_vs_oracle(xb, shape):
    print(f"case image shape={shape}", flush=True)
    run_case(xb, shape)


def test_image_forward_matches_the_staged_pipeline(xb):
    """The one-kernel pass and input_prepare + conv2d_fwd give the same dots and the same output
    to within the two paths' different fp32 summation orders for K."""
    shape = (2, 3, 45, 83, 6, 3, 1)
    print(f"case image-vs-staged shape={shape}", flush=True)
    s, dI, Wpk, alpha, out, dot = run_case(xb, shape, "staged")
    Ipk, K, _ = xb.xnor_input_prepare(dI, s)
    out_s, dot_s = xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, want_dot=True)
    torch.cuda.synchronize()
    assert torch.equal(dot, dot_s)
    a, b = out.cpu().numpy().astype(np.float64), out_s.cpu().numpy().astype(np.float64)
    assert (np.abs(a - b) <= 1e-5 * np.abs(b)).all()


@pytest.mark.parametrize("side", [256, 512, 1024, 2048])
def test_paper_sizes(xb, side):
    """Tables I-III: one channel, one 3x3 filter, zero padding, square images."""
    print(f"case image paper size={side}", flush=True)
    run_case(xb, (1, 1, side, side, 1, 3, 1), "paper")


def test_two_calls_in_a_row_do_not_interfere(xb):
    a = run_case(xb, (1, 1, 128, 128, 1, 3, 1), "first")
    b = run_case(xb, (1, 2, 50, 50, 3, 5, 2), "second")
    a2 = run_case(xb, (1, 1, 128, 128, 1, 3, 1), "first")
    assert torch.equal(a[4], a2[4]) and torch.equal(a[5], a2[5])


@pytest.mark.parametrize("full", [
    (1, 5, 16, 16, 1, 3, 3, 1, 1, 1, 1),      # too many channels
    (1, 1, 16, 16, 1, 3, 5, 1, 1, 1, 2),      # not square
    (1, 1, 16, 16, 1, 4, 4, 1, 1, 1, 1),      # even kernel
    (1, 1, 16, 16, 1, 9, 9, 1, 1, 4, 4),      # kernel too large
])
def test_shapes_the_kernel_does_not_take(xb, full):
    s = xb.Shape(*full)
    assert not xb.xnor_forward_image_supported(s)
    I = torch.zeros((s.N, s.C, s.H, s.W), dtype=torch.float32, device="cuda")
    Wpk = torch.zeros((s.F, s.kh, s.kw, 1), dtype=torch.int32, device="cuda")
    alpha = torch.ones((s.F,), dtype=torch.float32, device="cuda")
    with pytest.raises(xb.XnorError) as e:
        xb.xnor_forward_image(I, Wpk, alpha, s)
    assert e.value.status == xb.E_UNSUPPORTED
