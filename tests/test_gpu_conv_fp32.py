"""xnor_conv2d_fp32_fwd (the real-valued convolution that Table I, Sec. IV, compares the XNOR
convolution with) against the oracle.

The output is a signed sum of products, so its rounding error scales with the sum of their
magnitudes, not with the (possibly cancelled) result: the bar is |got - ref| <= 1e-5 * S,
S = sum |I * Wt| over the output's in-image terms (the oracle returns it), which still exposes a
single dropped or doubled term at every size tested (one term of kh*kw*C <= 6272 is >= 1.6e-4 of S
on average).  Outputs whose window is all padding are exactly 0.  The RMS bar keeps coarser
arithmetic (bf16, fp16, tf32 products) out.
"""
import zlib

import numpy as np
import pytest
import torch

import oracle
from paper_2007_14178_amd.workloads import LAYERS, make_input, make_weights, random_layer

pytestmark = pytest.mark.gpu
RTOL = 1e-5


@pytest.fixture(scope="module")
def xb():
    from paper_2007_14178_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


_CACHE: dict = {}


def oracle_conv(key, I, Wt, osh):
    if key not in _CACHE:
        if len(_CACHE) > 3:
            _CACHE.clear()
        O, S = oracle.conv_fp32(I, Wt, osh, want_scale=True)
        _CACHE[key] = (O.astype(np.float64), S)
    return _CACHE[key]


def check(xb, full, I, Wt, algo, key):
    s = xb.Shape(*full)
    O_ref, S = oracle_conv(key, I, Wt, oracle.Shape(*full))
    algo_id = {"auto": xb.ALGO_AUTO, "direct": xb.ALGO_DIRECT, "mfma": xb.ALGO_MFMA}[algo]
    try:
        out = xb.xnor_conv2d_fp32_fwd(dev(I), dev(Wt), s, algo=algo_id)
    except xb.XnorError as e:
        if e.status == xb.E_UNSUPPORTED and algo == "mfma":
            pytest.skip("the matrix-core kernel does not take this shape")
        raise
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert got.shape == O_ref.shape
    bar = RTOL * S
    err = np.abs(got - O_ref)
    assert (err <= bar).all(), f"{(err > bar).sum()} of {err.size} outside the bar; worst err/bar {np.nanmax(err / np.maximum(bar, 1e-300)):.3g}"
    assert np.sqrt((err ** 2).mean()) <= 2e-7 * np.sqrt((S ** 2).mean()) + 1e-30
    return out


#        N   C   H   W   F  kh kw sh sw ph pw
SHAPES = [
    (1, 1, 5, 5, 1, 1, 1, 1, 1, 0, 0),
    (1, 3, 9, 11, 2, 3, 3, 1, 1, 1, 1),
    (3, 31, 8, 7, 5, 3, 3, 1, 1, 1, 1),
    (2, 32, 13, 13, 33, 3, 3, 1, 1, 1, 1),
    (1, 33, 10, 12, 7, 2, 2, 1, 1, 0, 0),
    (2, 40, 9, 9, 4, 3, 3, 1, 1, 3, 2),          # windows that are all padding
    (3, 65, 12, 20, 9, 3, 5, 2, 1, 1, 2),        # strides, non-square kernel, channel tail
    (2, 96, 27, 27, 200, 5, 5, 1, 1, 2, 2),      # two filter groups, the second partly empty; weights beyond 64 KB of LDS
    (1, 70, 15, 17, 130, 1, 7, 1, 3, 0, 3),
    (2, 20, 30, 300, 3, 3, 3, 1, 1, 1, 1),       # rows wider than a workgroup's pixels
    (1, 130, 14, 14, 40, 7, 7, 1, 1, 3, 3),      # 49 taps: more weights per chunk than LDS holds (matrix-core kernel refuses)
    (5, 256, 14, 14, 130, 3, 3, 2, 2, 1, 1),
    (1, 8, 64, 64, 16, 3, 3, 1, 1, 1, 1),
    (3, 129, 31, 1, 2, 1, 1, 1, 2, 3, 0),        # staged rows one value wide
    (2, 40, 1, 1, 5, 1, 1, 1, 1, 0, 0),          # a staged plane of a single value
    (1, 24, 6, 500, 5, 3, 3, 1, 1, 1, 1),        # rows too wide to be fetched a chunk ahead
    (1, 1, 256, 256, 1, 3, 3, 1, 1, 1, 1),       # the paper's own workload shape (Table I)
    (2, 3, 17, 19, 3, 5, 5, 2, 1, 2, 2),         # few channels: four outputs per thread, ragged row ends, row stride 2
    (1, 4, 30, 44, 2, 7, 7, 1, 1, 3, 3),         # the same with the widest window and 16-byte stores
    (1, 2, 9, 8, 5, 3, 1, 1, 1, 0, 0),           # one-column window
]


@pytest.mark.parametrize("algo", ["direct", "mfma", "auto"])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_fp32_shapes_vs_oracle(xb, shape, algo):
    print(f"case conv_fp32 shape={shape} algo={algo}", flush=True)
    rng = np.random.default_rng(zlib.crc32(("conv_fp32" + str(shape)).encode()))
    _, I, Wt = random_layer(rng, "t", *shape)
    check(xb, shape, I, Wt, algo, shape)


@pytest.mark.parametrize("name", ["c1", "c2_k3", "c2_k5", "c3_s2", "c4_conv2", "c4_conv4", "c5"])
def test_conv_fp32_benchmark_layers_two_images(xb, name):
    L = LAYERS[name]
    n = min(L.N, 2)
    print(f"case conv_fp32 layer={name} images={n}", flush=True)
    I, Wt = make_input(L, n), make_weights(L)
    full = (n, L.C, L.H, L.W, L.F, L.kh, L.kw, L.sh, L.sw, L.ph, L.pw)
    out_m = check(xb, full, I, Wt, "mfma", name)
    out_d = check(xb, full, I, Wt, "direct", name)
    # the two kernels differ only in summation order
    assert torch.allclose(out_m, out_d, rtol=0, atol=float(2e-5 * out_d.abs().max()))


def test_conv_fp32_on_binary_data_equals_the_xnor_dot(xb):
    """With I and Wt in {+1,-1} every partial sum is a small integer, exact in fp32: the result is the
    dot product that the XNOR kernels compute from the packed signs of the same tensors."""
    shape = (2, 64, 20, 20, 40, 3, 3, 1, 1, 1, 1)
    print(f"case conv_fp32-binary shape={shape}", flush=True)
    rng = np.random.default_rng(12)
    _, I, Wt = random_layer(rng, "t", *shape)
    I = np.where(I >= 0, 1.0, -1.0).astype(np.float32)
    Wt = np.where(Wt >= 0, 1.0, -1.0).astype(np.float32)
    s = xb.Shape(*shape)
    dI, dW = dev(I), dev(Wt)
    Ipk, K, _ = xb.xnor_input_prepare(dI, s)
    Wpk, alpha, _ = xb.xnor_filter_prepare(dW)
    _, dot = xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, want_dot=True)
    for algo in (xb.ALGO_MFMA, xb.ALGO_DIRECT):
        out = xb.xnor_conv2d_fp32_fwd(dI, dW, s, algo=algo)
        torch.cuda.synchronize()
        assert torch.equal(out, dot.to(torch.float32))
    assert np.array_equal(dot.cpu().numpy(), oracle.dot(I, Wt, oracle.Shape(*shape)))


def test_conv_fp32_full_size_c5_sampled(xb):
    """The benchmark layer at its full batch, in the launch configuration bench.py times: whole
    images sampled across the batch against the oracle."""
    L = LAYERS["c5"]
    print("case conv_fp32 c5 full batch", flush=True)
    I, Wt = make_input(L), make_weights(L)
    s = xb.Shape(L.N, L.C, L.H, L.W, L.F, L.kh, L.kw, L.sh, L.sw, L.ph, L.pw)
    out = xb.xnor_conv2d_fp32_fwd(dev(I), dev(Wt), s)
    torch.cuda.synchronize()
    pick = [0, 1, 63, 126, 127]
    osh = oracle.Shape(len(pick), L.C, L.H, L.W, L.F, L.kh, L.kw, L.sh, L.sw, L.ph, L.pw)
    O_ref, S = oracle.conv_fp32(I[pick], Wt, osh, want_scale=True)
    got = out[pick].cpu().numpy().astype(np.float64)
    err = np.abs(got - O_ref.astype(np.float64))
    assert (err <= RTOL * S).all()
    assert np.sqrt((err ** 2).mean()) <= 2e-7 * np.sqrt((S ** 2).mean())
