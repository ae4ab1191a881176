"""GPU parity: every C-ABI call against the CPU oracle, element by element, same seeded inputs.

Bars: packed words and raw binary dot products bit-exact; A, K, alpha and the fp32 output within
1e-5 relative of the oracle (one fp32 subnormal spacing where that is larger; exactly 0 where the
oracle is 0).
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


def assert_rel(got: np.ndarray, ref: np.ndarray, what: str, floor=2.0 ** -149):
    got = got.astype(np.float64); ref = ref.astype(np.float64)
    assert got.shape == ref.shape, what
    err = np.abs(got - ref)
    # below fp32's normal range the spacing of representable values (2^-149) exceeds RTOL*|ref|:
    # there the bar is the nearest representable value (for the output: see out_floor)
    bad = err > np.maximum(RTOL * np.abs(ref), floor)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside {RTOL} rel; worst {err.max()}"
    assert np.array_equal(got == 0, ref == 0), f"{what}: zero pattern differs"


def out_floor(dot_ref: np.ndarray, alpha_ref: np.ndarray) -> np.ndarray:
    """Absolute error the fp32 pipeline can make on an output that lies in fp32's subnormal range,
    in the oracle's own terms: K reaches the convolution as an fp32 value (half a subnormal spacing
    off, times |dot| * alpha), K * alpha is rounded again (half a spacing, times |dot|) and so is
    the product.  In the normal range the relative bar is far larger than this."""
    d = np.abs(dot_ref.astype(np.float64))
    a = alpha_ref.astype(np.float64)[None, :, None, None]
    return (0.5 * d * (a + 1.0) + 1.0) * 2.0 ** -149


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def words(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def run_pipeline(xb, layer, I, Wt, algo, want_dot=True):
    s = xb.Shape(layer.N, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw,
                 layer.sh, layer.sw, layer.ph, layer.pw)
    dI, dW = dev(I), dev(Wt)
    Ipk = xb.xnor_binarize_pack(dI)
    Wpk = xb.xnor_binarize_pack(dW)
    K, A = xb.xnor_scale_K(dI, s)
    alpha = xb.xnor_alpha(dW)
    out, dot = xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, want_dot=want_dot, algo=algo)
    torch.cuda.synchronize()
    return s, Ipk, Wpk, K, A, alpha, out, dot


def oshape(layer):
    return oracle.Shape(layer.N, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw,
                        layer.sh, layer.sw, layer.ph, layer.pw)


_ORACLE_CACHE: dict = {}


def oracle_results(key, layer, I, Wt):
    """The oracle's outputs for one case, computed once and reused across the kernel variants."""
    if key not in _ORACLE_CACHE:
        if len(_ORACLE_CACHE) > 4:
            _ORACLE_CACHE.clear()
        _ORACLE_CACHE[key] = (oracle.pack(I), oracle.pack(Wt), oracle.channel_mean_abs(I),
                              *oracle.forward(I, Wt, oshape(layer)))
    return _ORACLE_CACHE[key]


def check_all(xb, layer, I, Wt, algo, key):
    s, Ipk, Wpk, K, A, alpha, out, dot = run_pipeline(xb, layer, I, Wt, algo)
    Ipk_ref, Wpk_ref, A_ref, d_ref, K_ref, a_ref, O_ref = oracle_results(key, layer, I, Wt)
    assert np.array_equal(words(Ipk), Ipk_ref), "Ipk"
    assert np.array_equal(words(Wpk), Wpk_ref), "Wpk"
    assert_rel(A.cpu().numpy(), A_ref, "A")
    assert_rel(K.cpu().numpy(), K_ref, "K")
    assert_rel(alpha.cpu().numpy(), a_ref, "alpha")
    assert np.array_equal(dot.cpu().numpy(), d_ref), "dot"
    assert_rel(out.cpu().numpy(), O_ref, "out", out_floor(d_ref, a_ref))
    # the one-pass variants of the pre-stages give the same packed words, A, K and alpha
    Ipk2, K2, A2 = xb.xnor_input_prepare(dev(I), s)
    Wpk2, alpha2, M2 = xb.xnor_filter_prepare(dev(Wt))
    torch.cuda.synchronize()
    assert np.array_equal(words(Ipk2), Ipk_ref), "Ipk (one pass)"
    assert np.array_equal(words(Wpk2), Wpk_ref), "Wpk (one pass)"
    assert_rel(A2.cpu().numpy(), A_ref, "A (one pass)")
    assert_rel(K2.cpu().numpy(), K_ref, "K (one pass)")
    assert_rel(alpha2.cpu().numpy(), a_ref, "alpha (one pass)")
    assert_rel(M2.cpu().numpy(), oracle.channel_mean_abs(Wt), "mean_c |Wt| (one pass)")


ALGOS = ["direct", "tiled", "mfma", "mfma_bands", "auto"]   # innermost parameter, so one oracle run serves all


def algo_id(xb, name):
    return {"auto": xb.ALGO_AUTO, "direct": xb.ALGO_DIRECT, "tiled": xb.ALGO_TILED, "mfma": xb.ALGO_MFMA,
            "mfma_bands": xb.ALGO_MFMA_BANDS}[name]


def run_or_skip(xb, layer, I, Wt, algo, key):
    try:
        check_all(xb, layer, I, Wt, algo_id(xb, algo), key)
    except xb.XnorError as e:
        if e.status == xb.E_UNSUPPORTED and algo in ("tiled", "mfma", "mfma_bands"):
            pytest.skip(f"{algo} does not take this shape")
        raise


# adversarial shapes: channel tails, even / non-square kernels, strides, oversized padding, odd batch,
# sizes that are not multiples of any tile, F not a multiple of the filter tile
#        N   C   H   W   F  kh kw sh sw ph pw
SHAPES = [
    (1, 1, 5, 5, 1, 1, 1, 1, 1, 0, 0),
    (1, 3, 9, 11, 2, 3, 3, 1, 1, 1, 1),
    (3, 31, 8, 7, 5, 3, 3, 1, 1, 1, 1),
    (2, 32, 13, 13, 33, 3, 3, 1, 1, 1, 1),
    (1, 33, 10, 12, 7, 2, 2, 1, 1, 0, 0),
    (2, 63, 17, 9, 17, 5, 5, 1, 1, 2, 2),
    (1, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1),
    (3, 65, 12, 20, 9, 3, 5, 2, 1, 1, 2),
    (1, 96, 27, 27, 40, 5, 5, 1, 1, 2, 2),
    (2, 128, 28, 28, 48, 3, 3, 2, 2, 1, 1),
    (1, 70, 15, 14, 6, 7, 7, 3, 3, 3, 3),
    (2, 40, 9, 9, 4, 3, 3, 1, 1, 3, 2),        # padding larger than k//2: some windows all padding
    (5, 256, 14, 14, 70, 3, 3, 1, 1, 1, 1),
    (1, 512, 28, 28, 96, 3, 3, 1, 1, 1, 1),
    (2, 128, 56, 56, 32, 7, 7, 1, 1, 3, 3),
    (1, 160, 6, 40, 130, 1, 3, 1, 2, 0, 1),
    (1, 1, 256, 256, 1, 3, 3, 1, 1, 1, 1),     # the paper's own workload shape (Tables I-III): one channel, one filter
    (2, 3, 300, 200, 2, 3, 3, 1, 1, 1, 1),     # rows wider than one band of the matrix-core kernel
]


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_shapes_vs_oracle(xb, shape, algo):
    rng = np.random.default_rng(zlib.crc32(str(shape).encode()))
    layer, I, Wt = random_layer(rng, "t", *shape)
    print(f"case shape={shape} algo={algo}", flush=True)
    run_or_skip(xb, layer, I, Wt, algo, shape)


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("name", ["c1", "c2_k3", "c2_k5", "c2_k7", "c3_s1", "c3_s2",
                                  "c4_conv2", "c4_conv3", "c4_conv4", "c4_conv5", "c5"])
def test_benchmark_layers_reduced_batch(xb, name, algo):
    """Each benchmark layer at its real C, H, W, F, kernel, stride and pad, on its first images
    (batch cut so that the oracle finishes in seconds)."""
    full = LAYERS[name]
    n = 1 if full.binary_macs // full.N > 1.5e9 else min(full.N, 2)
    layer = full.with_batch(n)
    I, Wt = make_input(full, n), make_weights(full)
    print(f"case layer={name} N={n} algo={algo}", flush=True)
    run_or_skip(xb, layer, I, Wt, algo, name)


def test_special_values(xb):
    """+0.0, -0.0, denormals, infinities -> sign by (x >= 0); NaN -> -1."""
    vals = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-39, -1e-39, np.inf, -np.inf, np.nan, -np.nan, 2.0, -2.0],
                    dtype=np.float32)
    x = np.tile(vals, 96 * 3)[: 96 * 3 * 4].reshape(1, 96, 3, 4).copy()
    got = words(xb.xnor_binarize_pack(dev(x)))
    assert np.array_equal(got, oracle.pack(x))


def test_determinism(xb):
    layer = LAYERS["c3_s1"].with_batch(4)
    I, Wt = make_input(LAYERS["c3_s1"], 4), make_weights(LAYERS["c3_s1"])
    for algo in ("direct", "tiled", "mfma", "mfma_bands"):
        try:
            r1 = run_pipeline(xb, layer, I, Wt, algo_id(xb, algo))
            r2 = run_pipeline(xb, layer, I, Wt, algo_id(xb, algo))
        except xb.XnorError as e:
            if e.status == xb.E_UNSUPPORTED:
                continue
            raise
        for a, b in zip(r1[1:], r2[1:]):
            assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def test_outputs_do_not_spill(xb):
    """Canary words around every output buffer stay untouched."""
    shape = (2, 70, 11, 13, 37, 3, 3, 1, 1, 1, 1)
    rng = np.random.default_rng(7)
    layer, I, Wt = random_layer(rng, "canary", *shape)
    s = xb.Shape(*shape)
    OH, OW = xb.xnor_out_dim(s)
    dI, dW = dev(I), dev(Wt)
    G = 64

    def guarded(n, dtype):
        buf = torch.full((n + 2 * G,), -7777, dtype=dtype, device="cuda")
        return buf, buf[G:G + n]

    for algo in ("direct", "tiled", "mfma", "mfma_bands"):
        bI, vI = guarded(s.N * s.H * s.W * s.Cw, torch.int32)
        bW, vW = guarded(s.F * s.kh * s.kw * s.Cw, torch.int32)
        bA, vA = guarded(s.N * s.H * s.W, torch.float32)
        bK, vK = guarded(s.N * OH * OW, torch.float32)
        ba, va = guarded(s.F, torch.float32)
        bo, vo = guarded(s.N * s.F * OH * OW, torch.float32)
        bd, vd = guarded(s.N * s.F * OH * OW, torch.int32)
        Ipk = xb.xnor_binarize_pack(dI, vI.view(s.N, s.H, s.W, s.Cw))
        Wpk = xb.xnor_binarize_pack(dW, vW.view(s.F, s.kh, s.kw, s.Cw))
        K, _ = xb.xnor_scale_K(dI, s, vA.view(s.N, s.H, s.W), vK.view(s.N, OH, OW))
        al = xb.xnor_alpha(dW, va)
        try:
            xb.xnor_conv2d_fwd(Ipk, Wpk, K, al, s, vo.view(s.N, s.F, OH, OW), vd.view(s.N, s.F, OH, OW),
                               algo=algo_id(xb, algo))
        except xb.XnorError as e:
            if e.status == xb.E_UNSUPPORTED:
                continue
            raise
        torch.cuda.synchronize()
        for b in (bI, bW, bA, bK, ba, bo, bd):
            assert (b[:G] == -7777).all() and (b[-G:] == -7777).all()
        assert np.array_equal(vd.cpu().numpy().reshape(s.N, s.F, OH, OW), oracle.dot(I, Wt, oshape(layer)))


def test_dot_null_gives_same_out(xb):
    layer = LAYERS["c1"]
    I, Wt = make_input(layer), make_weights(layer)
    for algo in ("direct", "tiled", "mfma", "mfma_bands"):
        try:
            a = run_pipeline(xb, layer, I, Wt, algo_id(xb, algo), want_dot=True)
            b = run_pipeline(xb, layer, I, Wt, algo_id(xb, algo), want_dot=False)
        except xb.XnorError as e:
            if e.status == xb.E_UNSUPPORTED:
                continue
            raise
        assert b[-1] is None and torch.equal(a[-2], b[-2])


@pytest.mark.parametrize("misalign", [0, 1])
@pytest.mark.parametrize("shape", [(3, 64, 28, 28, 160, 3, 3, 1, 1, 1, 1),     # last band ragged (84 of 252 pixels)
                                   (5, 64, 14, 14, 150, 3, 3, 1, 1, 1, 1),     # bands span images; last filter tile partial
                                   (2, 32, 30, 30, 64, 5, 5, 1, 1, 2, 2),      # 240-pixel bands, half a tile idle
                                   (2, 64, 26, 12, 96, 3, 3, 1, 1, 1, 1),      # 12-pixel rows
                                   (2, 64, 56, 56, 64, 3, 3, 2, 2, 1, 1),      # stride 2
                                   (2, 64, 13, 13, 64, 3, 3, 1, 1, 1, 1),      # 169 pixels per plane: no quads
                                   (44, 32, 28, 28, 512, 3, 3, 1, 1, 1, 1),    # more than one round of items, ragged end
                                   (130, 64, 14, 14, 256, 3, 3, 1, 1, 1, 1)],  # one round, bands span images
                         ids=lambda s: "x".join(map(str, s)) if isinstance(s, tuple) else str(s))
def test_fp32_output_alone_through_16_byte_stores(xb, shape, misalign):
    """Without the dot output, where planes and bands are whole groups of four pixels, `out` is
    16-byte aligned and the layer is more than one round of the kernel's items, the matrix-core
    kernel writes four consecutive pixels per lane through an LDS transposition.  Same bits as the run that also returns the dot products (whose stores are one
    pixel per lane), the oracle's values, every element written and nothing outside the tensor;
    with `out` only 4-byte aligned the one-pixel path runs and gives the same."""
    print(f"case quad stores shape={shape} misalign={misalign}", flush=True)
    rng = np.random.default_rng(zlib.crc32(repr(shape).encode()))
    layer, I, Wt = random_layer(rng, "t", *shape)
    s = xb.Shape(*shape)
    OH, OW = xb.xnor_out_dim(s)
    dI, dW = dev(I), dev(Wt)
    Ipk, Wpk = xb.xnor_binarize_pack(dI), xb.xnor_binarize_pack(dW)
    K, _ = xb.xnor_scale_K(dI, s)
    alpha = xb.xnor_alpha(dW)
    try:
        ref, dot = xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, want_dot=True, algo=xb.ALGO_MFMA)
    except xb.XnorError as e:
        if e.status == xb.E_UNSUPPORTED:
            pytest.skip("shape not taken by the matrix-core kernel")
        raise
    n = s.N * s.F * OH * OW
    guard = 4096
    buf = torch.full((n + 2 * guard + 4,), float("nan"), dtype=torch.float32, device="cuda")
    out = buf[guard + misalign:guard + misalign + n].view(s.N, s.F, OH, OW)
    assert out.data_ptr() % 16 == 4 * misalign
    xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, out=out, algo=xb.ALGO_MFMA)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(out).any())
    assert bool(torch.isnan(buf[:guard + misalign]).all()) and bool(torch.isnan(buf[guard + misalign + n:]).all())
    assert torch.equal(out, ref)
    d_ref, _, a_ref, O_ref = oracle.forward(I, Wt, oshape(layer))
    assert np.array_equal(dot.cpu().numpy(), d_ref)
    assert_rel(out.cpu().numpy(), O_ref, "out", out_floor(d_ref, a_ref))


@pytest.mark.parametrize("shape", [(2, 96, 27, 27, 40, 5, 5, 1, 1, 2, 2), (3, 512, 14, 14, 130, 3, 3, 1, 1, 1, 1),
                                   (1, 64, 32, 32, 64, 3, 3, 2, 2, 1, 1)], ids=lambda s: "x".join(map(str, s)))
def test_two_call_matrix_core_path(xb, shape):
    """xnor_filter_expand once, xnor_conv2d_fwd_expanded on two different inputs: bit-exact dots and
    outputs within 1e-5 of the oracle, and the same bits as the one-call form."""
    print(f"case two-call shape={shape}", flush=True)
    rng = np.random.default_rng(zlib.crc32(("two" + str(shape)).encode()))
    layer, I1, Wt = random_layer(rng, "t", *shape)
    _, I2, _ = random_layer(rng, "t", *shape)
    s = xb.Shape(*shape)
    Wpk, alpha, _ = xb.xnor_filter_prepare(dev(Wt))
    ws = xb.xnor_filter_expand(Wpk, s)
    for I in (I1, I2):
        Ipk, K, _ = xb.xnor_input_prepare(dev(I), s)
        out, dot = xb.xnor_conv2d_fwd_expanded(Ipk, ws, K, alpha, s, want_dot=True)
        out1, dot1 = xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, want_dot=True, algo=xb.ALGO_MFMA)
        torch.cuda.synchronize()
        d_ref, K_ref, a_ref, O_ref = oracle.forward(I, Wt, oshape(layer))
        assert np.array_equal(dot.cpu().numpy(), d_ref), "dot"
        assert_rel(out.cpu().numpy(), O_ref, "out", out_floor(d_ref, a_ref))
        assert torch.equal(out, out1) and torch.equal(dot, dot1)


@pytest.mark.parametrize("shape", [(3, 40, 148, 150), (1, 33, 260, 256), (2, 8, 200, 180), (1, 100, 256, 257)],
                         ids=lambda s: "x".join(map(str, s)))
def test_input_prepare_on_large_images(xb, shape):
    """xnor_input_prepare on images of 40 000 to 66 000 pixels, with channel tails and a ragged last
    block (H*W odd and even)."""
    N, C, H, W = shape
    print(f"case input_prepare shape={shape}", flush=True)
    rng = np.random.default_rng(zlib.crc32(("prep" + str(shape)).encode()))
    _, I, _ = random_layer(rng, "t", N, C, H, W, 1, 3, 3, 1, 1, 1, 1)
    s = xb.Shape(N, C, H, W, 1, 3, 3, 1, 1, 1, 1)
    Ipk, K, A = xb.xnor_input_prepare(dev(I), s)
    torch.cuda.synchronize()
    assert np.array_equal(words(Ipk), oracle.pack(I)), "Ipk"
    assert_rel(A.cpu().numpy(), oracle.channel_mean_abs(I), "A")
    assert_rel(K.cpu().numpy(), oracle.scale_K(I, oracle.Shape(N, C, H, W, 1, 3, 3, 1, 1, 1, 1)), "K")


@pytest.mark.parametrize("offset_words", [1, 2, 3])
def test_buffers_that_are_only_4_or_8_byte_aligned(xb, offset_words):
    """Every buffer placed 4, 8 or 12 bytes past a 16-byte boundary: the kernels that use 16-byte
    accesses on aligned operands must take their narrower paths and give the same results."""
    shape = (2, 128, 28, 28, 64, 3, 3, 1, 1, 1, 1)
    print(f"case misaligned offset={offset_words} words shape={shape}", flush=True)
    rng = np.random.default_rng(offset_words)
    layer, I, Wt = random_layer(rng, "t", *shape)
    s = xb.Shape(*shape)
    OH, OW = xb.xnor_out_dim(s)

    def shifted(n, dtype):
        buf = torch.empty((n + 4,), dtype=dtype, device="cuda")
        v = buf[offset_words:offset_words + n]
        assert v.data_ptr() % 16 == 4 * offset_words
        return v

    dI = shifted(I.size, torch.float32); dI.copy_(torch.from_numpy(I).reshape(-1).cuda()); dI = dI.view(I.shape)
    dW = shifted(Wt.size, torch.float32); dW.copy_(torch.from_numpy(Wt).reshape(-1).cuda()); dW = dW.view(Wt.shape)
    Ipk = shifted(s.N * s.H * s.W * s.Cw, torch.int32).view(s.N, s.H, s.W, s.Cw)
    Wpk = shifted(s.F * 9 * s.Cw, torch.int32).view(s.F, 3, 3, s.Cw)
    A = shifted(s.N * s.H * s.W, torch.float32).view(s.N, s.H, s.W)
    K = shifted(s.N * OH * OW, torch.float32).view(s.N, OH, OW)
    alpha = shifted(s.F, torch.float32)
    M = shifted(s.F * 9, torch.float32).view(s.F, 3, 3)
    out = shifted(s.N * s.F * OH * OW, torch.float32).view(s.N, s.F, OH, OW)
    dot = shifted(s.N * s.F * OH * OW, torch.int32).view(s.N, s.F, OH, OW)
    xb.xnor_input_prepare(dI, s, Ipk, A, K)
    xb.xnor_filter_prepare(dW, Wpk, M, alpha)
    d_ref, K_ref, a_ref, O_ref = oracle.forward(I, Wt, oshape(layer))
    assert np.array_equal(words(Ipk), oracle.pack(I)) and np.array_equal(words(Wpk), oracle.pack(Wt))
    assert_rel(K.cpu().numpy(), K_ref, "K")
    assert_rel(alpha.cpu().numpy(), a_ref, "alpha")
    for algo in ("direct", "tiled", "mfma", "mfma_bands"):
        out.zero_(); dot.zero_()
        xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, out=out, dot=dot, algo=algo_id(xb, algo))
        torch.cuda.synchronize()
        assert np.array_equal(dot.cpu().numpy(), d_ref), f"dot ({algo})"
        assert_rel(out.cpu().numpy(), O_ref, f"out ({algo})", out_floor(d_ref, a_ref))
    # the Binary-Weight-Network layer on the same shifted buffers
    O_bwn, S = oracle.bwn(I, Wt, oshape(layer), want_scale=True)
    xb.xnor_bwn_conv2d_fwd(dI, Wpk, alpha, s, out=out)
    torch.cuda.synchronize()
    err = np.abs(out.cpu().numpy().astype(np.float64) - O_bwn)
    assert (err <= RTOL * a_ref.astype(np.float64)[None, :, None, None] * S[:, None]).all()


@pytest.mark.parametrize("shape", [(2, 64, 28, 28, 96, 3, 3, 1, 1, 1, 1), (3, 40, 13, 13, 130, 5, 5, 1, 1, 2, 2),
                                   (2, 32, 20, 31, 33, 3, 3, 2, 2, 1, 1), (1, 128, 9, 9, 64, 3, 3, 1, 1, 3, 3)],
                         ids=lambda s: "x".join(map(str, s)))
def test_conv_that_forms_K_itself(xb, shape):
    """xnor_input_prepare without K + xnor_conv2d_fwd_expanded given A: the workgroups form K from A
    with the box filter's own arithmetic, so dots and outputs equal the staged path bit for bit."""
    print(f"case K-from-A shape={shape}", flush=True)
    rng = np.random.default_rng(zlib.crc32(("fromA" + str(shape)).encode()))
    layer, I, Wt = random_layer(rng, "t", *shape)
    s = xb.Shape(*shape)
    dI = dev(I)
    Ipk, none, A = xb.xnor_input_prepare(dI, s, want_K=False)
    assert none is None
    Wpk, alpha, _ = xb.xnor_filter_prepare(dev(Wt))
    ws = xb.xnor_filter_expand(Wpk, s)
    out, dot = xb.xnor_conv2d_fwd_expanded(Ipk, ws, None, alpha, s, want_dot=True, A=A)
    _, K, _ = xb.xnor_input_prepare(dI, s)
    out2, dot2 = xb.xnor_conv2d_fwd_expanded(Ipk, ws, K, alpha, s, want_dot=True)
    torch.cuda.synchronize()
    assert torch.equal(dot, dot2) and torch.equal(out, out2)
    d_ref, K_ref, a_ref, O_ref = oracle.forward(I, Wt, oshape(layer))
    assert np.array_equal(dot.cpu().numpy(), d_ref)
    assert_rel(out.cpu().numpy(), O_ref, "out", out_floor(d_ref, a_ref))


@pytest.mark.parametrize("shape", [(90, 256, 28, 28, 70, 3, 3, 1, 1, 1, 1),      # one launch for both sides
                                   (84, 288, 28, 28, 33, 5, 5, 1, 1, 2, 2),      # the same, ragged blocks, channel words 9
                                   (2, 64, 13, 13, 40, 3, 3, 1, 1, 1, 1),        # one launch, one-pixel input pass (H*W odd)
                                   (3, 96, 27, 27, 130, 5, 5, 1, 1, 2, 2),       # the same, three channel words, partial filter tile
                                   (2, 16, 20, 20, 5, 9, 9, 1, 1, 4, 4),         # more taps than a one-slice block has threads: separate launches
                                   (1, 1552, 256, 256, 3, 3, 3, 1, 1, 1, 1)],    # 49 channel words: the four-pixel pass's LDS would pass 64 KB
                         ids=lambda s: "x".join(map(str, s)))
def test_prepare_both_sides_in_one_call(xb, shape):
    """xnor_prepare gives bit for bit what xnor_input_prepare and xnor_filter_prepare give."""
    print(f"case prepare shape={shape}", flush=True)
    rng = np.random.default_rng(zlib.crc32(("both" + str(shape)).encode()))
    layer, I, Wt = random_layer(rng, "t", *shape)
    s = xb.Shape(*shape)
    dI, dW = dev(I), dev(Wt)
    Ipk, K, A, Wpk, alpha, M = xb.xnor_prepare(dI, dW, s)
    Ipk2, K2, A2 = xb.xnor_input_prepare(dI, s)
    Wpk2, alpha2, M2 = xb.xnor_filter_prepare(dW)
    torch.cuda.synchronize()
    for a, b, what in ((Ipk, Ipk2, "Ipk"), (K, K2, "K"), (A, A2, "A"), (Wpk, Wpk2, "Wpk"), (alpha, alpha2, "alpha"), (M, M2, "M")):
        assert torch.equal(a, b), what
    assert np.array_equal(words(Ipk), oracle.pack(I)) and np.array_equal(words(Wpk), oracle.pack(Wt))
    assert_rel(alpha.cpu().numpy(), oracle.alpha(Wt), "alpha")
    assert_rel(A.cpu().numpy(), oracle.channel_mean_abs(I), "A")
    _, none, _, _, _, _ = xb.xnor_prepare(dI, dW, s, want_K=False)
    assert none is None
    # with a workspace the expanded filters are what xnor_filter_expand makes of Wpk, byte for byte
    nbytes = xb.xnor_conv2d_workspace_bytes(s)
    assert nbytes > 0
    ws = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device="cuda")
    xb.xnor_prepare(dI, dW, s, workspace=ws)
    ws2 = xb.xnor_filter_expand(Wpk2, s, workspace=torch.full((nbytes,), 0x5A, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert torch.equal(ws, ws2)


def test_step_replays_from_a_hip_graph(xb):
    """The library allocates nothing and records no memset, so a whole step can be captured into a HIP
    graph: every replay (with eager work and synchronisations in between) equals the eager result."""
    shape = (8, 256, 28, 28, 96, 3, 3, 1, 1, 1, 1)
    print(f"case graph shape={shape}", flush=True)
    rng = np.random.default_rng(5)
    layer, I, Wt = random_layer(rng, "t", *shape)
    s = xb.Shape(*shape)
    OH, OW = xb.xnor_out_dim(s)
    dI, dW = dev(I), dev(Wt)
    ws = torch.empty((xb.xnor_conv2d_workspace_bytes(s),), dtype=torch.uint8, device="cuda")
    Ipk, _, A, Wpk, alpha, M = xb.xnor_prepare(dI, dW, s, want_K=False, workspace=ws)
    out = torch.empty((s.N, s.F, OH, OW), dtype=torch.float32, device="cuda")
    Opk = torch.empty((s.N, OH, OW, (s.F + 31) // 32), dtype=torch.int32, device="cuda")
    A_next = torch.empty((s.N, OH, OW), dtype=torch.float32, device="cuda")
    cws = torch.empty((xb.xnor_conv2d_chain_workspace_bytes(s),), dtype=torch.uint8, device="cuda")
    img_out = torch.empty((1, 1, 64, 64), dtype=torch.float32, device="cuda")
    img = torch.randn((1, 1, 64, 64), device="cuda")
    ishape = xb.Shape(1, 1, 64, 64, 1, 3, 3, 1, 1, 1, 1)
    iW = torch.randn((1, 1, 3, 3), device="cuda")
    iWpk, ialpha, _ = xb.xnor_filter_prepare(iW)
    bwn_out = torch.empty_like(out)

    def step():
        xb.xnor_prepare(dI, dW, s, Ipk, A, None, Wpk, M, alpha, want_K=False, workspace=ws)
        xb.xnor_conv2d_fwd_expanded(Ipk, ws, None, alpha, s, out=out, A=A)
        xb.xnor_conv2d_fwd_chain(Ipk, Wpk, None, alpha, s, Opk, A_next, cws, A=A)
        xb.xnor_forward_image(img, iWpk, ialpha, ishape, out=img_out)
        xb.xnor_bwn_conv2d_fwd(dI, Wpk, alpha, s, out=bwn_out)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (out, Opk, A_next, img_out, bwn_out)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for t in (out, A_next, img_out, bwn_out):
            t.fill_(float("nan"))
        Opk.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, what in zip((out, Opk, A_next, img_out, bwn_out), want, ("out", "Opk", "A_next", "image", "bwn")):
            assert torch.equal(got, ref), f"replay {rep}: {what}"
    d_ref, _, a_ref, O_ref = oracle.forward(I, Wt, oshape(layer))
    assert_rel(out.cpu().numpy(), O_ref, "out", out_floor(d_ref, a_ref))


def test_two_streams_at_once(xb):
    """Every call enqueues on the caller's stream and the library keeps no state between calls: two
    different layers issued alternately on two streams (default priority), several rounds in flight
    at once, give the bits that each gives alone."""
    shapes = [(6, 256, 28, 28, 130, 3, 3, 1, 1, 1, 1), (9, 96, 27, 27, 64, 5, 5, 1, 1, 2, 2)]
    print(f"case two streams shapes={shapes}", flush=True)
    jobs = []
    for k, shape in enumerate(shapes):
        rng = np.random.default_rng(70 + k)
        layer, I, Wt = random_layer(rng, "t", *shape)
        s = xb.Shape(*shape)
        OH, OW = xb.xnor_out_dim(s)
        dI, dW = dev(I), dev(Wt)
        ws = torch.empty((xb.xnor_conv2d_workspace_bytes(s),), dtype=torch.uint8, device="cuda")
        Ipk, _, A, Wpk, alpha, M = xb.xnor_prepare(dI, dW, s, want_K=False, workspace=ws)
        out = torch.empty((s.N, s.F, OH, OW), dtype=torch.float32, device="cuda")
        bwn = torch.empty_like(out)

        def run(dI=dI, dW=dW, s=s, Ipk=Ipk, A=A, Wpk=Wpk, M=M, alpha=alpha, ws=ws, out=out, bwn=bwn):
            xb.xnor_prepare(dI, dW, s, Ipk, A, None, Wpk, M, alpha, want_K=False, workspace=ws)
            xb.xnor_conv2d_fwd_expanded(Ipk, ws, None, alpha, s, out=out, A=A)
            xb.xnor_bwn_conv2d_fwd(dI, Wpk, alpha, s, out=bwn)

        run()
        torch.cuda.synchronize()
        jobs.append((run, out, bwn, out.clone(), bwn.clone(), torch.cuda.Stream()))
    for run, out, bwn, *_ in jobs:
        out.fill_(float("nan")); bwn.fill_(float("nan"))
    torch.cuda.synchronize()
    for _ in range(4):
        for run, *_, stream in jobs:
            with torch.cuda.stream(stream):
                run()
    torch.cuda.synchronize()
    for k, (run, out, bwn, out_ref, bwn_ref, _) in enumerate(jobs):
        assert torch.equal(out, out_ref), f"layer {k}: out"
        assert torch.equal(bwn, bwn_ref), f"layer {k}: bwn"
