"""xnor_bwn_conv2d_fwd (Binary-Weight-Network layer, Sec. II-A Eq. 1) against the oracle.

The output is a signed sum of real values, so its rounding error scales with the sum of the
magnitudes under the window, not with the (possibly cancelled) result: the bar is
|got - ref| <= 1e-5 * alpha[f] * S, S = sum |I| over the output's in-image taps (the oracle returns
it), which still exposes a single dropped or doubled term at every size tested (one term of
kh*kw*C <= 6272 is >= 1.6e-4 of S on average).  Outputs whose window is all padding are exactly 0.
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


def oracle_bwn(key, I, Wt, osh):
    if key not in _CACHE:
        if len(_CACHE) > 3:
            _CACHE.clear()
        O, S = oracle.bwn(I, Wt, osh, want_scale=True)
        _CACHE[key] = (O.astype(np.float64), S, oracle.alpha(Wt).astype(np.float64))
    return _CACHE[key]


def check(xb, full, I, Wt, algo, key):
    s = xb.Shape(*full)
    O_ref, S, a = oracle_bwn(key, I, Wt, oracle.Shape(*full))
    Wpk, alpha, _ = xb.xnor_filter_prepare(dev(Wt))
    algo_id = {"auto": xb.ALGO_AUTO, "direct": xb.ALGO_DIRECT, "mfma": xb.ALGO_MFMA, "split": xb.ALGO_MFMA_SPLIT}[algo]
    try:
        out = xb.xnor_bwn_conv2d_fwd(dev(I), Wpk, alpha, s, algo=algo_id)
    except xb.XnorError as e:
        if e.status == xb.E_UNSUPPORTED and algo in ("mfma", "split"):
            pytest.skip("the matrix-core kernel does not take this shape")
        raise
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert got.shape == O_ref.shape
    bar = RTOL * a[None, :, None, None] * S[:, None]
    if algo in ("split", "auto"):
        # the three-term bf16 kernel flushes terms below the normal range: at most 2^-125 per input value
        bar = bar + a[None, :, None, None] * (full[1] * full[5] * full[6]) * 2.0 ** -125
    err = np.abs(got - O_ref)
    assert (err <= bar).all(), f"{(err > bar).sum()} of {err.size} outside the bar; worst err/bar {np.nanmax(err / np.maximum(bar, 1e-300)):.3g}"
    # typical accuracy is far inside the bar: a coarser arithmetic (bf16, fp16) would not pass this
    assert np.sqrt((err ** 2).mean()) <= 2e-7 * np.sqrt(((a[None, :, None, None] * S[:, None]) ** 2).mean()) + 1e-30
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
    (2, 96, 27, 27, 200, 5, 5, 1, 1, 2, 2),      # two filter groups, the second partly empty
    (1, 70, 15, 17, 130, 1, 7, 1, 3, 0, 3),
    (2, 20, 30, 300, 3, 3, 3, 1, 1, 1, 1),       # rows wider than a workgroup's pixels
    (1, 130, 14, 14, 40, 7, 7, 1, 1, 3, 3),
    (5, 256, 14, 14, 130, 3, 3, 2, 2, 1, 1),
    (1, 8, 64, 64, 16, 3, 3, 1, 1, 1, 1),
    (3, 129, 31, 1, 2, 1, 1, 1, 2, 3, 0),        # staged rows one value wide (a divisor of 1 in the staging index math)
    (2, 40, 1, 1, 5, 1, 1, 1, 1, 0, 0),          # a staged plane of a single value
    (1, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3),      # a ResNet-style first layer
    (1, 24, 6, 500, 5, 3, 3, 1, 1, 1, 1),        # rows too wide to be fetched a chunk ahead
]


@pytest.mark.parametrize("algo", ["direct", "mfma", "split", "auto"])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_bwn_shapes_vs_oracle(xb, shape, algo):
    print(f"case bwn shape={shape} algo={algo}", flush=True)
    rng = np.random.default_rng(zlib.crc32(("bwn" + str(shape)).encode()))
    _, I, Wt = random_layer(rng, "t", *shape)
    check(xb, shape, I, Wt, algo, shape)


@pytest.mark.parametrize("name", ["c1", "c2_k3", "c2_k7", "c3_s2", "c4_conv2", "c4_conv4", "c5"])
def test_bwn_benchmark_layers_two_images(xb, name):
    L = LAYERS[name]
    n = min(L.N, 2)
    print(f"case bwn layer={name} images={n}", flush=True)
    I, Wt = make_input(L, n), make_weights(L)
    full = (n, L.C, L.H, L.W, L.F, L.kh, L.kw, L.sh, L.sw, L.ph, L.pw)
    out_m = check(xb, full, I, Wt, "mfma", name)
    out_s = check(xb, full, I, Wt, "split", name)
    out_d = check(xb, full, I, Wt, "direct", name)
    # the kernels differ only in summation order
    assert torch.allclose(out_m, out_d, rtol=0, atol=float(2e-5 * out_d.abs().max()))
    assert torch.allclose(out_s, out_d, rtol=0, atol=float(2e-5 * out_d.abs().max()))


def test_bwn_tiny_inputs_stay_within_the_flush_floor(xb):
    """Inputs at the bottom of the fp32 range: the fp32 kernels carry them exactly (sums of a few
    denormals are exact), the three-term bf16 kernel may flush each term below 2^-126."""
    shape = (2, 20, 9, 9, 12, 3, 3, 1, 1, 1, 1)
    print(f"case bwn-tiny shape={shape}", flush=True)
    rng = np.random.default_rng(5)
    _, I, Wt = random_layer(rng, "t", *shape)
    tiny = np.float32(1e-41) * rng.integers(-200, 200, size=I.shape).astype(np.float32)
    small = (I * np.float32(1e-35)).astype(np.float32)
    I = np.where(rng.random(I.shape) < 0.5, tiny, small).astype(np.float32)
    s = xb.Shape(*shape)
    O_ref, S = oracle.bwn(I, Wt, oracle.Shape(*shape), want_scale=True)
    a = oracle.alpha(Wt).astype(np.float64)
    Wpk, alpha, _ = xb.xnor_filter_prepare(dev(Wt))
    nred = shape[1] * shape[5] * shape[6]
    for algo, floor in ((xb.ALGO_DIRECT, 0.0), (xb.ALGO_MFMA, 0.0), (xb.ALGO_MFMA_SPLIT, 2.0 ** -125), (xb.ALGO_AUTO, 2.0 ** -125)):
        out = xb.xnor_bwn_conv2d_fwd(dev(I), Wpk, alpha, s, algo=algo)
        torch.cuda.synchronize()
        err = np.abs(out.cpu().numpy().astype(np.float64) - O_ref.astype(np.float64))
        bar = RTOL * a[None, :, None, None] * S[:, None] + a[None, :, None, None] * nred * floor + 2.0 ** -149
        assert (err <= bar).all(), f"algo {algo}: {(err > bar).sum()} of {err.size} outside the bar"


def test_bwn_on_binary_input_equals_the_xnor_path(xb):
    """With I in {+1,-1} the sums are small integers, exact in fp32: the result is dot * alpha, where
    dot is what the XNOR kernels compute from the packed signs of the same tensors."""
    shape = (2, 64, 20, 20, 40, 3, 3, 1, 1, 1, 1)
    print(f"case bwn-binary shape={shape}", flush=True)
    rng = np.random.default_rng(11)
    _, I, Wt = random_layer(rng, "t", *shape)
    I = np.where(I >= 0, 1.0, -1.0).astype(np.float32)
    s = xb.Shape(*shape)
    dI = dev(I)
    Wpk, alpha, _ = xb.xnor_filter_prepare(dev(Wt))
    Ipk, K, _ = xb.xnor_input_prepare(dI, s)
    _, dot = xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, want_dot=True)
    for algo in (xb.ALGO_DIRECT, xb.ALGO_MFMA, xb.ALGO_MFMA_SPLIT):
        out = xb.xnor_bwn_conv2d_fwd(dI, Wpk, alpha, s, algo=algo)
        torch.cuda.synchronize()
        assert torch.equal(out, dot.float() * alpha[None, :, None, None])


def test_measurement_probes_run(xb):
    """The probes of bench.py --peaks: each enqueues its kernel and reports the work it issued."""
    print("case probes", flush=True)
    sink_f = torch.zeros((4,), dtype=torch.float32, device="cuda")
    sink_i = torch.zeros((4,), dtype=torch.int32, device="cuda")
    assert xb.xnor_probe_mfma_fp4(256, 10, sink_f) == 256 * 4 * 10 * 8 * 32 * 32 * 64 * 2
    assert xb.xnor_probe_mfma_bf16(256, 10, False, sink_f) == 256 * 4 * 10 * 6 * 32 * 32 * 16 * 2
    assert xb.xnor_probe_mfma_bf16(256, 10, True, sink_f) == 256 * 4 * 10 * 6 * 32 * 32 * 16 * 2
    assert xb.xnor_probe_xor_popcount(256, 10, sink_i) == 256 * 256 * 10 * 8 * 32
    src = torch.arange(1 << 16, dtype=torch.float32, device="cuda")
    dst = torch.zeros_like(src)
    assert xb.xnor_probe_copy(src, dst) == src.numel() * 4
    assert xb.xnor_probe_read(src, sink_i) == src.numel() * 4
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert float(sink_f.abs().sum()) == 0.0 and int(sink_i.abs().sum()) == 0
    # the store probe writes every byte of its destination and nothing else, and reports a time per wave
    wgs, reps = 8, 2
    n = wgs * reps * 32768
    for wide in (False, True):
        for loop in (0, 1, 2):
            buf = torch.full((n + 64,), float("nan"), dtype=torch.float32, device="cuda")
            cycles = torch.zeros((wgs, 4), dtype=torch.int64, device="cuda")
            xb.xnor_probe_store_beside_mfma(wgs, reps, wide, loop, buf[:n], cycles, sink_f)
            torch.cuda.synchronize()
            assert not bool(torch.isnan(buf[:n]).any()) and bool(torch.isnan(buf[n:]).all())
            assert bool((cycles > 0).all())
    assert float(sink_f.abs().sum()) == 0.0
