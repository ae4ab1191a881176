"""Pins for the CPU oracle (no GPU needed).

The oracle is the reference every GPU result is compared with, so it is pinned here to things
other than itself: hand-worked fixtures, the XNOR-popcount identity (Sec. III-A step 1c: a 0 bit
stands for -1, hence dot = 2*popcount(XNOR) - N), a differently-structured brute-force evaluation,
closed forms, invariants, library special cases and distribution statistics.  Shapes are chosen
asymmetric (H != W, kh != kw, sh != sw, ph != pw) so that a transposed index fails.
"""
import itertools
import json
import os
import zlib

import numpy as np
import pytest
import torch

import oracle
from oracle import Shape

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")


def _h(s) -> int:
    return zlib.crc32(str(s).encode())


# ----------------------------------------------------------------------------------------------
# independent evaluations (numpy only; nothing below calls the oracle)
# ----------------------------------------------------------------------------------------------
def np_sign(x):
    """+1 where x >= 0 (so +0.0 and -0.0 give +1, NaN gives -1)."""
    return np.where(x >= 0, 1, -1).astype(np.int64)


def out_hw(s: Shape):
    return (s.H + 2 * s.ph - s.kh) // s.sh + 1, (s.W + 2 * s.pw - s.kw) // s.sw + 1


def brute_dot_im2col(I, Wt, s: Shape):
    """Materialise the zero-padded +-1/0 tensor, unfold it, one int64 matrix product."""
    OH, OW = out_hw(s)
    P = np.zeros((s.N, s.C, s.H + 2 * s.ph, s.W + 2 * s.pw), dtype=np.int64)
    P[:, :, s.ph:s.ph + s.H, s.pw:s.pw + s.W] = np_sign(I)
    cols = np.empty((s.N, OH, OW, s.C, s.kh, s.kw), dtype=np.int64)
    for oy in range(OH):
        for ox in range(OW):
            cols[:, oy, ox] = P[:, :, oy * s.sh:oy * s.sh + s.kh, ox * s.sw:ox * s.sw + s.kw]
    M = cols.reshape(s.N * OH * OW, -1) @ np_sign(Wt).reshape(s.F, -1).T
    return M.reshape(s.N, OH, OW, s.F).transpose(0, 3, 1, 2)


_POP8 = np.array([bin(i).count("1") for i in range(256)], dtype=np.int64)


def packed_popcount_dot(I, Wt, s: Shape):
    """Bits packed along channels into bytes; dot = 2*popcount(XNOR & valid) - N_valid per tap."""
    OH, OW = out_hw(s)
    bi = np.packbits(I >= 0, axis=1, bitorder="little")          # [N][Cb][H][W]
    bw = np.packbits(Wt >= 0, axis=1, bitorder="little")         # [F][Cb][kh][kw]
    Cb = bi.shape[1]
    tail = np.packbits(np.arange(Cb * 8) < s.C, bitorder="little")  # valid-channel mask per byte
    dot = np.zeros((s.N, s.F, OH, OW), dtype=np.int64)
    for ky, kx in itertools.product(range(s.kh), range(s.kw)):
        for oy in range(OH):
            iy = oy * s.sh - s.ph + ky
            if not 0 <= iy < s.H:
                continue
            for ox in range(OW):
                ix = ox * s.sw - s.pw + kx
                if not 0 <= ix < s.W:
                    continue
                a = bi[:, None, :, iy, ix]                        # [N][1][Cb]
                b = bw[None, :, :, ky, kx]                        # [1][F][Cb]
                xnor = (~(a ^ b)) & tail
                dot[:, :, oy, ox] += 2 * _POP8[xnor].sum(-1) - s.C
    return dot


def np_K(I, s: Shape):
    OH, OW = out_hw(s)
    A = np.abs(I.astype(np.float64)).sum(1) / s.C
    P = np.zeros((s.N, s.H + 2 * s.ph, s.W + 2 * s.pw))
    P[:, s.ph:s.ph + s.H, s.pw:s.pw + s.W] = A
    K = np.empty((s.N, OH, OW))
    for oy in range(OH):
        for ox in range(OW):
            K[:, oy, ox] = P[:, oy * s.sh:oy * s.sh + s.kh, ox * s.sw:ox * s.sw + s.kw].sum((1, 2))
    return K / (s.kh * s.kw)


def rand_case(seed, s: Shape, zeros=True):
    rng = np.random.default_rng(seed)
    I = rng.standard_normal((s.N, s.C, s.H, s.W)).astype(np.float32)
    Wt = rng.standard_normal((s.F, s.C, s.kh, s.kw)).astype(np.float32)
    if zeros:
        I[rng.random(I.shape) < 0.1] = 0.0
        I[rng.random(I.shape) < 0.05] = -0.0
        Wt[rng.random(Wt.shape) < 0.1] = -0.0
    return I, Wt


ASYM_SHAPES = [
    Shape(2, 3, 5, 7, 2, 3, 2, 1, 2, 1, 0),
    Shape(1, 33, 6, 4, 3, 2, 3, 2, 1, 0, 2),
    Shape(3, 65, 4, 9, 5, 1, 1, 1, 1, 0, 0),
    Shape(1, 7, 8, 5, 4, 5, 3, 3, 2, 3, 1),     # padding larger than k//2
    Shape(2, 96, 7, 7, 3, 7, 7, 1, 1, 3, 3),
    Shape(1, 1, 9, 11, 2, 3, 3, 1, 1, 1, 1),
]


# ----------------------------------------------------------------------------------------------
# 0. hand-worked fixtures
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", json.load(open(GOLDEN))["cases"], ids=lambda c: c["name"])
def test_hand_worked_fixture(case):
    s = Shape(**case["shape"])
    I = np.array(case["I"], dtype=np.float32)
    Wt = np.array(case["Wt"], dtype=np.float32)
    d, K, a, O = oracle.forward(I, Wt, s)
    assert np.array_equal(d, np.array(case["dot"], dtype=np.int32))
    assert np.array_equal(a, np.array(case["alpha"], dtype=np.float32))
    assert np.array_equal(oracle.channel_mean_abs(I), np.array(case["A"], dtype=np.float64))
    np.testing.assert_allclose(K, np.array(case["K"]), rtol=1e-7)
    np.testing.assert_allclose(O, np.array(case["O"]), rtol=2e-7)
    assert np.array_equal(oracle.bwn(I, Wt, s), np.array(case["O_bwn"], dtype=np.float32))
    assert np.array_equal(oracle.conv_fp32(I, Wt, s), np.array(case["O_conv"], dtype=np.float32))


# ----------------------------------------------------------------------------------------------
# 1. sign and the packed encoding
# ----------------------------------------------------------------------------------------------
def test_sign_special_values():
    x = np.array([0.0, -0.0, 1e-45, -1e-45, 3.0, -3.0, np.inf, -np.inf, np.nan], dtype=np.float32)
    assert oracle.sign(x).tolist() == [1, 1, 1, -1, 1, -1, 1, -1, -1]


@pytest.mark.parametrize("C", [1, 3, 31, 32, 33, 64, 65, 96])
def test_pack_encoding(C):
    rng = np.random.default_rng(C)
    x = rng.standard_normal((2, C, 3, 5)).astype(np.float32)
    x[rng.random(x.shape) < 0.1] = 0.0
    x[rng.random(x.shape) < 0.1] = -0.0
    p = oracle.pack(x)
    Cw = (C + 31) // 32
    assert p.shape == (2, 3, 5, Cw) and p.dtype == np.uint32
    # independent decode: bit j of word w is channel 32w+j; bits past C are zero
    bits = ((p[..., None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(2, 3, 5, Cw * 32)
    assert not bits[..., C:].any()
    assert np.array_equal(bits[..., :C].transpose(0, 3, 1, 2) == 1, x >= 0)
    # against numpy's own bit packer (little-endian bytes -> little-endian words)
    ref = np.packbits(np.pad(x >= 0, ((0, 0), (0, Cw * 32 - C), (0, 0), (0, 0))).transpose(0, 2, 3, 1),
                      axis=-1, bitorder="little").view("<u4")
    assert np.array_equal(p, ref)


# ----------------------------------------------------------------------------------------------
# 2. brute force / identity on small tensors
# ----------------------------------------------------------------------------------------------
def test_dot_exhaustive_tiny():
    """Every sign pattern of a 1x1x2x2 image against every 2x2 filter, pad 1."""
    s = Shape(1, 1, 2, 2, 1, 2, 2, 1, 1, 1, 1)
    for ibits in range(16):
        I = np.array([1.0 if ibits >> k & 1 else -1.0 for k in range(4)], np.float32).reshape(1, 1, 2, 2)
        for wbits in range(16):
            Wt = np.array([1.0 if wbits >> k & 1 else -1.0 for k in range(4)], np.float32).reshape(1, 1, 2, 2)
            assert np.array_equal(oracle.dot(I, Wt, s), brute_dot_im2col(I, Wt, s))


@pytest.mark.parametrize("s", ASYM_SHAPES, ids=str)
def test_dot_matches_bruteforce_and_popcount_identity(s):
    I, Wt = rand_case(_h(s), s)
    d = oracle.dot(I, Wt, s)
    assert d.dtype == np.int32
    assert np.array_equal(d, brute_dot_im2col(I, Wt, s))
    assert np.array_equal(d, packed_popcount_dot(I, Wt, s))


@pytest.mark.parametrize("s", ASYM_SHAPES, ids=str)
def test_K_alpha_out_match_numpy(s):
    I, Wt = rand_case(1 + _h(s), s)
    d, K, a, O = oracle.forward(I, Wt, s)
    Kref = np_K(I, s)
    aref = np.abs(Wt.astype(np.float64)).reshape(s.F, -1).sum(1) / (s.C * s.kh * s.kw)
    np.testing.assert_allclose(K, Kref, rtol=1e-7, atol=0)
    np.testing.assert_allclose(a, aref, rtol=1e-7, atol=0)
    Oref = brute_dot_im2col(I, Wt, s) * Kref[:, None] * aref[None, :, None, None]
    np.testing.assert_allclose(O, Oref, rtol=3e-7, atol=0)
    assert np.array_equal(O == 0, Oref == 0)


# ----------------------------------------------------------------------------------------------
# 3. closed forms (pin padding, K's border rule and K's stride together)
# ----------------------------------------------------------------------------------------------
def valid_taps(s: Shape):
    OH, OW = out_hw(s)
    vy = np.array([sum(0 <= oy * s.sh - s.ph + ky < s.H for ky in range(s.kh)) for oy in range(OH)])
    vx = np.array([sum(0 <= ox * s.sw - s.pw + kx < s.W for kx in range(s.kw)) for ox in range(OW)])
    return vy[:, None] * vx[None, :]


@pytest.mark.parametrize("s", [Shape(2, 5, 6, 6, 3, 3, 3, 1, 1, 1, 1), Shape(1, 40, 9, 7, 2, 5, 3, 2, 1, 2, 1),
                               Shape(1, 4, 5, 5, 2, 3, 3, 2, 2, 2, 2)], ids=str)
def test_closed_forms(s):
    v = valid_taps(s)
    ones_I = np.ones((s.N, s.C, s.H, s.W), np.float32)
    ones_W = np.ones((s.F, s.C, s.kh, s.kw), np.float32)
    d, K, a, O = oracle.forward(ones_I, ones_W, s)
    assert np.array_equal(d, np.broadcast_to(s.C * v, d.shape))
    assert np.array_equal(a, np.ones(s.F, np.float32))
    np.testing.assert_allclose(K, np.broadcast_to(v / (s.kh * s.kw), K.shape), rtol=1e-7)
    np.testing.assert_allclose(O, np.broadcast_to(s.C * v * v / (s.kh * s.kw), O.shape), rtol=2e-7)
    # 3x3, pad 1, stride 1: interior 9C, edge 4C, corner 16C/9
    if (s.kh, s.kw, s.ph, s.pw, s.sh, s.sw) == (3, 3, 1, 1, 1, 1):
        assert O[0, 0, 2, 2] == 9 * s.C and O[0, 0, 0, 2] == 4 * s.C
        assert O[0, 0, 0, 0] == np.float32(16 * s.C / 9)
    # all-minus-one filters flip the sign only
    d2 = oracle.dot(ones_I, -ones_W, s)
    assert np.array_equal(d2, -d)
    # I == 0 everywhere: every bit is +1, dot = sum of in-image filter signs, K = 0, O = 0
    rng = np.random.default_rng(5)
    Wt = rng.standard_normal(ones_W.shape).astype(np.float32)
    d0, K0, _, O0 = oracle.forward(np.zeros_like(ones_I), Wt, s)
    assert np.array_equal(d0, brute_dot_im2col(np.ones_like(ones_I), Wt, s))
    assert not K0.any() and not O0.any()


def test_1x1_kernel_is_per_pixel_channel_dot():
    s = Shape(2, 37, 4, 5, 3, 1, 1)
    I, Wt = rand_case(11, s)
    d, K, _, _ = oracle.forward(I, Wt, s)
    ref = np.einsum("nchw,fc->nfhw", np_sign(I), np_sign(Wt[:, :, 0, 0]))
    assert np.array_equal(d, ref)
    np.testing.assert_allclose(K, oracle.channel_mean_abs(I), rtol=1e-7)


# ----------------------------------------------------------------------------------------------
# 4. invariants
# ----------------------------------------------------------------------------------------------
def test_invariants():
    s = Shape(2, 19, 7, 6, 4, 3, 3, 1, 1, 1, 1)
    I, Wt = rand_case(21, s, zeros=False)
    d, K, a, O = oracle.forward(I, Wt, s)
    nv = s.C * valid_taps(s)
    assert (np.abs(d) <= nv).all() and ((d - nv) % 2 == 0).all()
    # negate one filter
    W2 = Wt.copy(); W2[1] = -W2[1]
    d2, _, a2, _ = oracle.forward(I, W2, s)
    assert np.array_equal(d2[:, 1], -d[:, 1]) and np.array_equal(np.delete(d2, 1, 1), np.delete(d, 1, 1))
    assert np.array_equal(a2, a)
    # negate the input (no zeros present)
    d3, K3, _, _ = oracle.forward(-I, Wt, s)
    assert np.array_equal(d3, -d) and np.array_equal(K3, K)
    # positive scalings touch only K resp. alpha (powers of two: exact)
    d4, K4, a4, _ = oracle.forward(4 * I, Wt, s)
    assert np.array_equal(d4, d) and np.array_equal(K4, 4 * K) and np.array_equal(a4, a)
    W5 = Wt.copy(); W5[2] *= 8
    d5, K5, a5, _ = oracle.forward(I, W5, s)
    assert np.array_equal(d5, d) and np.array_equal(K5, K)
    assert a5[2] == 8 * a[2] and np.array_equal(np.delete(a5, 2), np.delete(a, 2))
    # same channel permutation on both operands
    perm = np.random.default_rng(3).permutation(s.C)
    d6, K6, a6, _ = oracle.forward(I[:, perm], Wt[:, perm], s)
    assert np.array_equal(d6, d)
    np.testing.assert_allclose(K6, K, rtol=1e-6); np.testing.assert_allclose(a6, a, rtol=1e-6)
    # translation by one pixel moves interior outputs
    I7 = np.zeros_like(I); I7[..., 1:] = I[..., :-1]
    d7 = oracle.dot(I7, Wt, s)
    assert np.array_equal(d7[..., 2:-1], d[..., 1:-2])


def test_kernel_flip_is_not_applied():
    """Cross-correlation: filter tap (ky,kx) meets input (oy+ky, ox+kx), not the mirrored one."""
    s = Shape(1, 1, 3, 3, 1, 2, 2)
    I = -np.ones((1, 1, 3, 3), np.float32); I[0, 0, 0, 0] = 1
    Wt = -np.ones((1, 1, 2, 2), np.float32); Wt[0, 0, 0, 0] = 1
    d = oracle.dot(I, Wt, s)
    assert d[0, 0, 0, 0] == 4          # both + meet at output (0,0)
    assert d[0, 0, 1, 1] == 2          # a flipped kernel would give 4 here and 0... at (0,0)


# ----------------------------------------------------------------------------------------------
# 5. library special cases
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("s", ASYM_SHAPES + [Shape(2, 64, 32, 32, 8, 3, 3, 1, 1, 1, 1)], ids=str)
def test_against_torch_cpu(s):
    I, Wt = rand_case(31 + _h(s), s)
    d, K, a, _ = oracle.forward(I, Wt, s)
    tI, tW = torch.from_numpy(I), torch.from_numpy(Wt)
    one = torch.tensor(1.0)
    sI, sW = torch.where(tI >= 0, one, -one), torch.where(tW >= 0, one, -one)
    dref = torch.nn.functional.conv2d(sI, sW, stride=(s.sh, s.sw), padding=(s.ph, s.pw))
    assert np.array_equal(d, dref.numpy().astype(np.int32))
    if s.ph <= s.kh // 2 and s.pw <= s.kw // 2:       # avg_pool2d refuses larger padding
        Kref = torch.nn.functional.avg_pool2d(tI.double().abs().mean(1, keepdim=True), (s.kh, s.kw),
                                              (s.sh, s.sw), (s.ph, s.pw), count_include_pad=True)[:, 0]
        np.testing.assert_allclose(K, Kref.numpy(), rtol=1e-6)
    np.testing.assert_allclose(a, tW.double().abs().mean((1, 2, 3)).numpy(), rtol=1e-6)


# ----------------------------------------------------------------------------------------------
# 6. statistics of N(0,1) data
# ----------------------------------------------------------------------------------------------
def test_statistics():
    s = Shape(4, 64, 16, 16, 16, 3, 3, 1, 1, 0, 0)
    I, Wt = rand_case(41, s, zeros=False)
    d, K, a, _ = oracle.forward(I, Wt, s)
    n = s.C * 9
    assert abs(d.mean()) < 0.5
    assert abs(d.astype(np.float64).var() / n - 1) < 0.05
    assert abs(K.mean() / np.sqrt(2 / np.pi) - 1) < 0.01
    assert abs(a.mean() / np.sqrt(2 / np.pi) - 1) < 0.02


# ----------------------------------------------------------------------------------------------
# 7. one image of each benchmark layer: identity still holds at real channel counts
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["c1", "c3_s2", "c4_conv3"])
def test_benchmark_layer_one_image_identity(name):
    from paper_2007_14178_amd.workloads import LAYERS, make_input, make_weights
    L = LAYERS[name]
    F = 8
    s = Shape(1, L.C, L.H, L.W, F, L.kh, L.kw, L.sh, L.sw, L.ph, L.pw)
    I, Wt = make_input(L, 1), make_weights(L)[:F]
    d = oracle.dot(I, Wt, s)
    tI, tW = torch.from_numpy(I), torch.from_numpy(Wt)
    one = torch.tensor(1.0)
    dref = torch.nn.functional.conv2d(torch.where(tI >= 0, one, -one), torch.where(tW >= 0, one, -one),
                                      stride=(s.sh, s.sw), padding=(s.ph, s.pw))
    assert np.array_equal(d, dref.numpy().astype(np.int32))


# ----------------------------------------------------------------------------------------------
# 8. Binary-Weight-Network layer (Sec. II-A, Eq. 1): real input, sign weights, alpha
# ----------------------------------------------------------------------------------------------
def brute_bwn_im2col(I, Wt, s: Shape):
    """Zero-padded real tensor, unfolded, one float64 matrix product with the +-1 filters, then
    alpha = mean |Wt| per filter (nothing here calls the oracle)."""
    OH, OW = out_hw(s)
    P = np.zeros((s.N, s.C, s.H + 2 * s.ph, s.W + 2 * s.pw), dtype=np.float64)
    P[:, :, s.ph:s.ph + s.H, s.pw:s.pw + s.W] = I
    cols = np.empty((s.N, OH, OW, s.C, s.kh, s.kw), dtype=np.float64)
    for oy in range(OH):
        for ox in range(OW):
            cols[:, oy, ox] = P[:, :, oy * s.sh:oy * s.sh + s.kh, ox * s.sw:ox * s.sw + s.kw]
    M = cols.reshape(s.N * OH * OW, -1) @ np_sign(Wt).reshape(s.F, -1).T.astype(np.float64)
    a = np.abs(Wt.astype(np.float64)).reshape(s.F, -1).mean(1)
    return M.reshape(s.N, OH, OW, s.F).transpose(0, 3, 1, 2) * a[None, :, None, None]


def window_l1(I, s: Shape):
    return np_K(I, s) * (s.C * s.kh * s.kw)


@pytest.mark.parametrize("s", ASYM_SHAPES, ids=str)
def test_bwn_matches_bruteforce(s):
    I, Wt = rand_case(_h(("bwn", s)), s)
    O, S = oracle.bwn(I, Wt, s, want_scale=True)
    ref = brute_bwn_im2col(I, Wt, s)
    l1 = window_l1(I, s)
    np.testing.assert_allclose(S, l1, rtol=1e-12, atol=1e-300)
    # both sides sum in double; the only difference is the order and the final rounding to fp32
    assert (np.abs(O - ref) <= 2.0 ** -23 * np.abs(ref) + 1e-13 * l1[:, None]).all()


@pytest.mark.parametrize("s", ASYM_SHAPES, ids=str)
def test_bwn_against_torch_cpu(s):
    I, Wt = rand_case(_h(("bwn-torch", s)), s)
    B = torch.from_numpy(np.where(Wt >= 0, 1.0, -1.0))
    ref = torch.nn.functional.conv2d(torch.from_numpy(I.astype(np.float64)), B, stride=(s.sh, s.sw),
                                     padding=(s.ph, s.pw)).numpy()
    ref = ref * torch.from_numpy(Wt.astype(np.float64)).abs().mean((1, 2, 3)).numpy()[None, :, None, None]
    O = oracle.bwn(I, Wt, s)
    l1 = window_l1(I, s)
    assert (np.abs(O - ref) <= 2.0 ** -23 * np.abs(ref) + 1e-13 * l1[:, None]).all()


def test_bwn_on_binary_input_is_the_xnor_dot_times_alpha():
    """With I in {+1,-1} the real-input convolution is the sign convolution (Eq. 1 vs Eq. 11)."""
    s = Shape(2, 37, 6, 5, 4, 3, 2, 2, 1, 1, 1)
    I, Wt = rand_case(77, s, zeros=False)
    I = np.where(I >= 0, 1.0, -1.0).astype(np.float32)
    O = oracle.bwn(I, Wt, s)
    expect = oracle.dot(I, Wt, s).astype(np.float64) * oracle.alpha(Wt).astype(np.float64)[None, :, None, None]
    assert np.array_equal(O, expect.astype(np.float32))


def test_bwn_closed_forms_and_invariants():
    s = Shape(2, 5, 6, 7, 3, 3, 3, 1, 1, 1, 1)
    OH, OW = out_hw(s)
    ones_I = np.full((s.N, s.C, s.H, s.W), 2.5, dtype=np.float32)
    ones_W = np.ones((s.F, s.C, s.kh, s.kw), dtype=np.float32)
    v = np_K(np.ones_like(ones_I), s) * 9                      # number of in-image taps
    assert np.array_equal(oracle.bwn(ones_I, ones_W, s), np.broadcast_to((2.5 * s.C * v)[:, None], (s.N, s.F, OH, OW)).astype(np.float32))
    assert np.array_equal(oracle.bwn(ones_I, -3 * ones_W, s), (-3 * 2.5 * s.C * np.broadcast_to(v[:, None], (s.N, s.F, OH, OW))).astype(np.float32))
    I, Wt = rand_case(5, s)
    O = oracle.bwn(I, Wt, s).astype(np.float64)
    l1 = window_l1(I, s)[:, None]
    a = oracle.alpha(Wt).astype(np.float64)[None, :, None, None]
    tol = 2.0 ** -22 * np.abs(O) + 1e-12 * l1
    # negating a filter negates its plane; scaling a filter by c > 0 scales its plane by c
    Wt0 = Wt.copy(); Wt0[Wt0 == 0] = 0.25                      # sign(-0) = sign(+0) = +1 does not negate
    O0 = oracle.bwn(I, Wt0, s).astype(np.float64)
    W2 = Wt0.copy(); W2[1] = -W2[1]; W2[2] = 4 * W2[2]
    O2 = oracle.bwn(I, W2, s).astype(np.float64)
    assert (np.abs(O2[:, 0] - O0[:, 0]) <= tol[:, 0]).all()
    assert (np.abs(O2[:, 1] + O0[:, 1]) <= tol[:, 1]).all()
    assert (np.abs(O2[:, 2] - 4 * O0[:, 2]) <= 4 * tol[:, 2]).all()
    # linear in the input
    I2, _ = rand_case(6, s)
    lhs = oracle.bwn((2 * I + 0.5 * I2).astype(np.float32), Wt, s).astype(np.float64)
    rhs = 2 * O + 0.5 * oracle.bwn(I2, Wt, s).astype(np.float64)
    scale = a * (2 * l1 + 0.5 * window_l1(I2, s)[:, None])
    assert (np.abs(lhs - rhs) <= 2.0 ** -21 * scale).all()
    # |O| <= alpha * sum |I| over the window
    assert (np.abs(O) <= a * l1 * (1 + 1e-6)).all()


# ----------------------------------------------------------------------------------------------
# real-valued convolution (the float comparison of Table I)
# ----------------------------------------------------------------------------------------------
def window_l1_products(I, Wt, s: Shape):
    """sum |I * Wt| over each output's terms: unfold |I| and multiply by |Wt| (double)."""
    OH, OW = out_hw(s)
    P = np.zeros((s.N, s.C, s.H + 2 * s.ph, s.W + 2 * s.pw))
    P[:, :, s.ph:s.ph + s.H, s.pw:s.pw + s.W] = np.abs(I.astype(np.float64))
    cols = np.empty((s.N, OH, OW, s.C, s.kh, s.kw))
    for oy in range(OH):
        for ox in range(OW):
            cols[:, oy, ox] = P[:, :, oy * s.sh:oy * s.sh + s.kh, ox * s.sw:ox * s.sw + s.kw]
    M = cols.reshape(s.N * OH * OW, -1) @ np.abs(Wt.astype(np.float64)).reshape(s.F, -1).T
    return M.reshape(s.N, OH, OW, s.F).transpose(0, 3, 1, 2)


@pytest.mark.parametrize("s", ASYM_SHAPES, ids=str)
def test_conv_fp32_against_torch_cpu(s):
    """torch's fp64 conv2d is an independent library routine of the same definition."""
    I, Wt = rand_case(_h(("conv", s)), s)
    ref = torch.nn.functional.conv2d(torch.from_numpy(I.astype(np.float64)), torch.from_numpy(Wt.astype(np.float64)),
                                     stride=(s.sh, s.sw), padding=(s.ph, s.pw)).numpy()
    O, S = oracle.conv_fp32(I, Wt, s, want_scale=True)
    l1 = window_l1_products(I, Wt, s)
    np.testing.assert_allclose(S, l1, rtol=1e-12, atol=1e-300)
    # both sides sum in double; what differs is the order and the oracle's final rounding to fp32
    assert (np.abs(O - ref) <= 2.0 ** -23 * np.abs(ref) + 1e-13 * l1).all()


def test_conv_fp32_brute_force_tiny():
    """Every output of a tiny case from the definition, in exact rational arithmetic."""
    from fractions import Fraction
    s = Shape(2, 3, 4, 5, 2, 3, 2, 2, 1, 1, 1)
    I, Wt = rand_case(11, s)
    OH, OW = out_hw(s)
    O = oracle.conv_fp32(I, Wt, s)
    for n, f, oy, ox in itertools.product(range(s.N), range(s.F), range(OH), range(OW)):
        acc = Fraction(0)
        for c, ky, kx in itertools.product(range(s.C), range(s.kh), range(s.kw)):
            iy, ix = oy * s.sh - s.ph + ky, ox * s.sw - s.pw + kx
            if 0 <= iy < s.H and 0 <= ix < s.W:
                acc += Fraction(float(I[n, c, iy, ix])) * Fraction(float(Wt[f, c, ky, kx]))
        assert abs(float(O[n, f, oy, ox]) - float(acc)) <= 2.0 ** -23 * abs(float(acc)) + 1e-30


def test_conv_fp32_reduces_to_the_other_two_convolutions():
    """On +-1 inputs and weights it is the sign convolution (Eq. 11's first factor); with weights
    alpha * sign(W) it is the Binary-Weight-Network layer (Eq. 1)."""
    s = Shape(2, 37, 6, 5, 4, 3, 2, 2, 1, 1, 1)
    I, Wt = rand_case(78, s, zeros=False)
    Ib = np.where(I >= 0, 1.0, -1.0).astype(np.float32)
    Wb = np.where(Wt >= 0, 1.0, -1.0).astype(np.float32)
    assert np.array_equal(oracle.conv_fp32(Ib, Wb, s), oracle.dot(I, Wt, s).astype(np.float32))
    a = oracle.alpha(Wt)
    Wa = (Wb * a[:, None, None, None]).astype(np.float32)       # exact: +-alpha
    O = oracle.conv_fp32(I, Wa, s).astype(np.float64)
    B = oracle.bwn(I, Wt, s).astype(np.float64)
    assert (np.abs(O - B) <= 2.0 ** -22 * np.abs(B) + 1e-12).all()


def test_conv_fp32_closed_forms_and_invariants():
    s = Shape(2, 5, 6, 7, 3, 3, 3, 1, 1, 1, 1)
    OH, OW = out_hw(s)
    taps = np_K(np.ones((s.N, s.C, s.H, s.W), dtype=np.float32), s) * 9     # number of in-image taps
    cI = np.full((s.N, s.C, s.H, s.W), 2.5, dtype=np.float32)
    cW = np.full((s.F, s.C, s.kh, s.kw), -0.75, dtype=np.float32)
    want = np.broadcast_to((2.5 * -0.75 * s.C * taps)[:, None], (s.N, s.F, OH, OW)).astype(np.float32)
    assert np.array_equal(oracle.conv_fp32(cI, cW, s), want)
    # a filter that is 1 at one tap of one channel copies that channel, shifted (cross-correlation:
    # tap (ky, kx) reads the pixel at (oy - ph + ky, ox - pw + kx)); outside the image it reads zero
    I, Wt = rand_case(12, s)
    d = np.zeros_like(Wt); d[0, 3, 0, 2] = 1.0                   # filter 0: channel 3, tap (0, 2)
    O = oracle.conv_fp32(I, d, s)
    shifted = np.zeros((s.N, OH, OW), dtype=np.float32)
    shifted[:, 1:, :-1] = I[:, 3, :-1, 1:]
    assert np.array_equal(O[:, 0], shifted) and not O[:, 1:].any()
    # linear in the input and in the weights; filters are independent of each other
    I2, W2 = rand_case(13, s)
    l1 = window_l1_products(I, Wt, s) + window_l1_products(I2, Wt, s) + window_l1_products(I, W2, s)
    base = oracle.conv_fp32(I, Wt, s).astype(np.float64)
    lhs = oracle.conv_fp32((2 * I + 0.5 * I2).astype(np.float32), Wt, s).astype(np.float64)
    assert (np.abs(lhs - (2 * base + 0.5 * oracle.conv_fp32(I2, Wt, s))) <= 2.0 ** -20 * l1).all()
    lhs = oracle.conv_fp32(I, (Wt - 4 * W2).astype(np.float32), s).astype(np.float64)
    assert (np.abs(lhs - (base - 4 * oracle.conv_fp32(I, W2, s))) <= 2.0 ** -19 * l1).all()
    Wp = Wt[[2, 0, 1]]
    assert np.array_equal(oracle.conv_fp32(I, Wp, s), oracle.conv_fp32(I, Wt, s)[:, [2, 0, 1]])
    # transposing image and filter transposes the output (a swapped ky / kx index would not)
    st = Shape(s.N, s.C, s.W, s.H, s.F, s.kw, s.kh, s.sw, s.sh, s.pw, s.ph)
    Ot = oracle.conv_fp32(np.ascontiguousarray(I.transpose(0, 1, 3, 2)), np.ascontiguousarray(Wt.transpose(0, 1, 3, 2)), st)
    assert np.array_equal(Ot.transpose(0, 1, 3, 2), oracle.conv_fp32(I, Wt, s))
