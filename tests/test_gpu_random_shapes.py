"""Seeded random layer shapes through every form of the forward pass, against the oracle.

The hand-picked shapes of the other GPU tests aim at known edges; this sweep draws shapes the
author did not choose (channel counts around the word and chunk sizes, filter counts around the
tile sizes, kernel / stride / padding combinations, images narrower and wider than a tile) and
sends each through: the four separate calls with every convolution kernel, the fused step
(`xnor_prepare` with the expanded-filter workspace + the convolution that forms K itself), the
chained form, the Binary-Weight-Network layer and, where it takes the shape, the one-kernel image
pass.  Bars as everywhere: dots and packed words bit-exact, fp32 within 1e-5 relative (in fp32's
subnormal range: what the fp32 roundings of the pipeline amount to there), BWN within
1e-5 * alpha * sum|I|.
"""
import zlib

import numpy as np
import pytest
import torch

import oracle
from paper_2007_14178_amd.workloads import random_layer

pytestmark = pytest.mark.gpu
RTOL = 1e-5
N_CASES = 120


@pytest.fixture(scope="module")
def xb():
    from paper_2007_14178_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def assert_rel(got, ref, what, floor=2.0 ** -149):
    got = got.astype(np.float64); ref = ref.astype(np.float64)
    assert got.shape == ref.shape, what
    err = np.abs(got - ref)
    bad = err > np.maximum(RTOL * np.abs(ref), floor)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside {RTOL} rel; worst {err.max()}"
    assert np.array_equal(got == 0, ref == 0), f"{what}: zero pattern differs"


def out_floor(dot_ref, alpha_ref):
    """Absolute error the fp32 pipeline can make on an output that lies in fp32's subnormal range,
    in the oracle's own terms: K reaches the convolution as an fp32 value (half a subnormal spacing
    off, times |dot| * alpha), K * alpha is rounded again (half a spacing, times |dot|) and so is
    the product.  In the normal range the relative bar is far larger than this."""
    d = np.abs(dot_ref.astype(np.float64))
    a = alpha_ref.astype(np.float64)[None, :, None, None]
    return (0.5 * d * (a + 1.0) + 1.0) * 2.0 ** -149


def draw_shape(rng):
    """N, C, H, W, F, kh, kw, sh, sw, ph, pw with at least one output pixel."""
    pick = lambda xs: int(xs[rng.integers(0, len(xs))])
    while True:
        C = pick([1, 2, 3, 4, 7, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 160, 255, 256, 257, 300])
        F = pick([1, 2, 5, 31, 32, 33, 63, 64, 65, 127, 128, 129, 140, 200])
        kh, kw = pick([1, 2, 3, 3, 3, 5, 7]), pick([1, 2, 3, 3, 3, 5, 7])
        if rng.random() < 0.6:
            kw = kh
        sh, sw = pick([1, 1, 1, 2, 3]), pick([1, 1, 1, 2, 3])
        ph, pw = pick([0, 1, 1, 2, 3]), pick([0, 1, 1, 2, 3])
        H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
        if rng.random() < 0.15:
            W = int(rng.integers(100, 300))          # wider than one band of the matrix-core kernels
        N = int(rng.integers(1, 5))
        if H + 2 * ph < kh or W + 2 * pw < kw:
            continue
        OH, OW = (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1
        if N * C * H * W > 3_000_000 or N * F * OH * OW * C * kh * kw > 400_000_000:
            continue                                 # keeps the oracle at well under a second a case
        return (N, C, H, W, F, kh, kw, sh, sw, ph, pw)


def cases():
    rng = np.random.default_rng(2007_14178)
    return [draw_shape(rng) for _ in range(N_CASES)]


@pytest.mark.parametrize("shape", cases(), ids=lambda s: "x".join(map(str, s)))
def test_random_shape_all_forms(xb, shape):
    print(f"case random shape={shape}", flush=True)
    rng = np.random.default_rng(zlib.crc32(str(shape).encode()))
    layer, I, Wt = random_layer(rng, "r", *shape)
    s, osh = xb.Shape(*shape), oracle.Shape(*shape)
    d_ref, K_ref, a_ref, O_ref = oracle.forward(I, Wt, osh)
    Ipk_ref, Wpk_ref, A_ref = oracle.pack(I), oracle.pack(Wt), oracle.channel_mean_abs(I)
    dI, dW = dev(I), dev(Wt)

    # the four separate calls, every convolution kernel that takes the shape
    Ipk, Wpk = xb.xnor_binarize_pack(dI), xb.xnor_binarize_pack(dW)
    K, A = xb.xnor_scale_K(dI, s)
    alpha = xb.xnor_alpha(dW)
    torch.cuda.synchronize()
    assert np.array_equal(Ipk.cpu().numpy().view(np.uint32), Ipk_ref), "Ipk"
    assert np.array_equal(Wpk.cpu().numpy().view(np.uint32), Wpk_ref), "Wpk"
    assert_rel(A.cpu().numpy(), A_ref, "A")
    assert_rel(K.cpu().numpy(), K_ref, "K")
    assert_rel(alpha.cpu().numpy(), a_ref, "alpha")
    outs = {}
    for name, algo in (("direct", xb.ALGO_DIRECT), ("tiled", xb.ALGO_TILED), ("mfma", xb.ALGO_MFMA), ("auto", xb.ALGO_AUTO)):
        try:
            out, dot = xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, want_dot=True, algo=algo)
        except xb.XnorError as e:
            assert e.status == xb.E_UNSUPPORTED and name in ("tiled", "mfma"), (name, e)
            continue
        torch.cuda.synchronize()
        assert np.array_equal(dot.cpu().numpy(), d_ref), f"dot ({name})"
        assert_rel(out.cpu().numpy(), O_ref, f"out ({name})", out_floor(d_ref, a_ref))
        outs[name] = out
    # every kernel forms the output with the same expression from the same exact dot
    for name, out in outs.items():
        assert torch.equal(out, outs["direct"]), f"{name} and direct differ in bits"

    # the fused step: one prepare call (with the expanded filters where the matrix-core kernel takes
    # the shape), then the convolution that forms K from A
    nbytes = xb.xnor_conv2d_workspace_bytes(s)
    if nbytes > 0:
        ws = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
        Ipk2, K2, A2, Wpk2, alpha2, _ = xb.xnor_prepare(dI, dW, s, want_K=False, workspace=ws)
        out2, dot2 = xb.xnor_conv2d_fwd_expanded(Ipk2, ws, None, alpha2, s, want_dot=True, A=A2)
        torch.cuda.synchronize()
        assert K2 is None
        assert torch.equal(Ipk2, Ipk) and torch.equal(Wpk2, Wpk), "packed words (fused prepare)"
        assert np.array_equal(dot2.cpu().numpy(), d_ref), "dot (fused step)"
        assert_rel(out2.cpu().numpy(), O_ref, "out (fused step)", out_floor(d_ref, a_ref))

        # chained form: packed signs and channel mean of the output
        Opk, A_next = xb.xnor_conv2d_fwd_chain(Ipk, Wpk, None, alpha, s, A=A)
        torch.cuda.synchronize()
        assert np.array_equal(Opk.cpu().numpy().view(np.uint32), oracle.pack(O_ref)), "packed signs of the output"
        An_ref = oracle.channel_mean_abs(O_ref)
        got = A_next.cpu().numpy()
        # (the mean over the filters of errors that each stay inside out_floor, and its own rounding)
        assert_rel(got, An_ref, "channel mean of |out|", out_floor(d_ref, a_ref).mean(axis=1) + 2.0 ** -149)

    # Binary-Weight-Network layer
    O_b, S = oracle.bwn(I, Wt, osh, want_scale=True)
    for name, algo in (("direct", xb.ALGO_DIRECT), ("mfma", xb.ALGO_MFMA), ("split", xb.ALGO_MFMA_SPLIT), ("auto", xb.ALGO_AUTO)):
        try:
            ob = xb.xnor_bwn_conv2d_fwd(dI, Wpk, alpha, s, algo=algo)
        except xb.XnorError as e:
            assert e.status == xb.E_UNSUPPORTED and name in ("mfma", "split"), (name, e)
            continue
        torch.cuda.synchronize()
        err = np.abs(ob.cpu().numpy().astype(np.float64) - O_b.astype(np.float64))
        bar = RTOL * a_ref.astype(np.float64)[None, :, None, None] * S[:, None]
        if name in ("split", "auto"):
            # (the three-term bf16 kernel may flush a term below the normal range: 2^-125 per input value)
            bar = bar + a_ref.astype(np.float64)[None, :, None, None] * (shape[1] * shape[5] * shape[6]) * 2.0 ** -125
        assert (err <= bar).all(), f"bwn ({name}): {(err > bar).sum()} of {err.size} outside the bar"

    # the one-kernel image pass
    if xb.xnor_forward_image_supported(s):
        oi, di = xb.xnor_forward_image(dI, Wpk, alpha, s, want_dot=True)
        torch.cuda.synchronize()
        assert np.array_equal(di.cpu().numpy(), d_ref), "dot (image pass)"
        # (this kernel sums K in fp32: kw*C + kh roundings instead of one)
        assert_rel(oi.cpu().numpy(), O_ref, "out (image pass)", out_floor(d_ref, a_ref * (shape[6] * shape[1] + shape[5])))
