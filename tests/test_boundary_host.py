"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and turns bad arguments into status codes before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def xb():
    from paper_2007_14178_amd import binding
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "xnor.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(xnor_[A-Za-z0-9_]+)\s*\(", text)))


def test_header_symbols_exported(xb):
    names = declared_symbols()
    assert {"xnor_binarize_pack", "xnor_scale_K", "xnor_alpha", "xnor_conv2d_fwd"} <= set(names)
    raw = ctypes.CDLL(xb.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), f"{n} declared in xnor.h but not exported"


def test_out_dim_and_words(xb):
    assert xb.xnor_out_dim(xb.Shape(1, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1)) == (32, 32)
    assert xb.xnor_out_dim(xb.Shape(1, 128, 28, 28, 256, 3, 3, 2, 2, 1, 1)) == (14, 14)
    assert xb.xnor_out_dim(xb.Shape(1, 8, 7, 9, 2, 3, 5, 2, 3, 0, 1)) == (3, 3)
    assert [xb.xnor_packed_words(c) for c in (1, 31, 32, 33, 64, 65, 512)] == [1, 1, 1, 2, 2, 3, 16]
    with pytest.raises(xb.XnorError):
        xb.xnor_packed_words(0)


def test_strerror_covers_every_status(xb):
    seen = {xb.lib.xnor_strerror(s) for s in range(0, -7, -1)}
    assert len(seen) == 7 and all(seen)
    assert xb.lib.xnor_strerror(-99)


BAD_SHAPES = [
    dict(N=0), dict(C=0), dict(H=-1), dict(W=0), dict(F=0), dict(kh=0), dict(kw=-3), dict(sh=0), dict(sw=-1),
    dict(ph=-1), dict(pw=-1), dict(kh=40, ph=1), dict(kw=40, pw=0),
    dict(N=70000, H=300, W=300),                 # N*H*W past 31 bits
]


@pytest.mark.parametrize("bad", BAD_SHAPES, ids=str)
def test_bad_shapes_rejected(xb, bad):
    base = dict(N=2, C=64, H=32, W=32, F=8, kh=3, kw=3, sh=1, sw=1, ph=1, pw=1)
    base.update(bad)
    s = xb.Shape(**base)
    oh, ow = ctypes.c_int(), ctypes.c_int()
    assert xb.lib.xnor_out_dim(ctypes.byref(s.c()), ctypes.byref(oh), ctypes.byref(ow)) == xb.E_SHAPE
    fake = ctypes.c_void_p(0x1000)
    assert xb.lib.xnor_scale_K(fake, ctypes.byref(s.c()), fake, fake, None) == xb.E_SHAPE
    assert xb.lib.xnor_conv2d_fwd(fake, fake, fake, fake, ctypes.byref(s.c()), fake, None, None, 0, None) == xb.E_SHAPE
    assert xb.lib.xnor_conv2d_pick_algo(ctypes.byref(s.c()), 0) == xb.E_SHAPE
    nb = ctypes.c_size_t()
    assert xb.lib.xnor_conv2d_workspace_bytes(ctypes.byref(s.c()), ctypes.byref(nb)) == xb.E_SHAPE


def test_null_and_alignment_rejected(xb):
    s = xb.Shape(1, 64, 8, 8, 4, 3, 3, 1, 1, 1, 1)
    sp = ctypes.byref(s.c())
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1002)
    L = xb.lib
    assert L.xnor_binarize_pack(None, 1, 64, 8, 8, ok, None) == xb.E_NULL
    assert L.xnor_binarize_pack(ok, 1, 64, 8, 8, None, None) == xb.E_NULL
    assert L.xnor_binarize_pack(ok, 1, 0, 8, 8, ok, None) == xb.E_SHAPE
    assert L.xnor_binarize_pack(odd, 1, 64, 8, 8, ok, None) == xb.E_ALIGN
    assert L.xnor_binarize_pack(ok, 1, 64, 8, 8, odd, None) == xb.E_ALIGN
    assert L.xnor_scale_K(None, sp, ok, ok, None) == xb.E_NULL
    assert L.xnor_scale_K(ok, None, ok, ok, None) == xb.E_NULL
    assert L.xnor_scale_K(ok, sp, None, ok, None) == xb.E_NULL
    assert L.xnor_scale_K(ok, sp, ok, odd, None) == xb.E_ALIGN
    assert L.xnor_alpha(None, 4, 64, 3, 3, ok, None) == xb.E_NULL
    assert L.xnor_alpha(ok, 4, 64, 3, 0, ok, None) == xb.E_SHAPE
    assert L.xnor_alpha(ok, 4, 64, 3, 3, odd, None) == xb.E_ALIGN
    for k in range(6):
        args = [ok, ok, ok, ok, sp, ok]
        args[k] = None
        assert L.xnor_conv2d_fwd(*args, None, None, 0, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd(odd, ok, ok, ok, sp, ok, None, None, 0, None) == xb.E_ALIGN
    assert L.xnor_conv2d_fwd(ok, ok, ok, ok, sp, ok, odd, None, 0, None) == xb.E_ALIGN
    assert L.xnor_conv2d_fwd(ok, ok, ok, ok, sp, ok, None, ctypes.c_void_p(0x1008), 1 << 20, None) == xb.E_ALIGN
    assert L.xnor_conv2d_fwd_algo(ok, ok, ok, ok, sp, ok, None, None, 0, 99, None) == xb.E_UNSUPPORTED
    # the matrix-core kernel refuses to run without its workspace; AUTO then picks another kernel
    assert L.xnor_conv2d_fwd_algo(ok, ok, ok, ok, sp, ok, None, None, 0, xb.ALGO_MFMA, None) == xb.E_WORKSPACE
    assert L.xnor_conv2d_fwd_algo(ok, ok, ok, ok, sp, ok, None, ok, 16, xb.ALGO_MFMA, None) == xb.E_WORKSPACE
    need = xb.xnor_conv2d_workspace_bytes(s)
    assert need > 0 and need % 1024 == 0
    assert xb.xnor_conv2d_pick_algo(s, need) == xb.ALGO_MFMA
    assert xb.xnor_conv2d_pick_algo(s, need - 1) != xb.ALGO_MFMA
    # the form with the workspace in the library's static array: argument checks come before any HIP call
    assert L.xnor_conv2d_fwd_static(None, ok, ok, ok, sp, ok, None, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd_static(ok, ok, ok, ok, sp, odd, None, None) == xb.E_ALIGN
    big = xb.Shape(1, 2048, 14, 14, 1024, 3, 3, 1, 1, 1, 1)
    assert xb.xnor_conv2d_workspace_bytes(big) > xb.STATIC_SCRATCH_BYTES
    assert L.xnor_conv2d_fwd_static(ok, ok, ok, ok, ctypes.byref(big.c()), ok, None, None) == xb.E_WORKSPACE
    # the two-call form of the matrix-core path
    assert L.xnor_filter_expand(None, sp, ok, need, None) == xb.E_NULL
    assert L.xnor_filter_expand(ok, sp, None, need, None) == xb.E_NULL
    assert L.xnor_filter_expand(ok, sp, ctypes.c_void_p(0x1008), need, None) == xb.E_ALIGN
    assert L.xnor_filter_expand(ok, sp, ok, need - 1, None) == xb.E_WORKSPACE
    # (Ipk, workspace, bytes, K, A, alpha, shape, out, dot, stream): exactly one of K, A
    assert L.xnor_conv2d_fwd_expanded(ok, None, need, ok, None, ok, sp, ok, None, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd_expanded(ok, ok, need, None, None, ok, sp, ok, None, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd_expanded(ok, ok, need, ok, ok, ok, sp, ok, None, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd_expanded(ok, ok, need - 1, ok, None, ok, sp, ok, None, None) == xb.E_WORKSPACE
    assert L.xnor_conv2d_fwd_expanded(ok, ok, need - 1, None, ok, ok, sp, ok, None, None) == xb.E_WORKSPACE
    assert L.xnor_conv2d_fwd_expanded(odd, ok, need, ok, None, ok, sp, ok, None, None) == xb.E_ALIGN
    assert L.xnor_conv2d_fwd_expanded(ok, ok, need, None, odd, ok, sp, ok, None, None) == xb.E_ALIGN
    # chained form: (Ipk, Wpk or NULL, K, A, alpha, shape, Opk, A_next, workspace, bytes, stream)
    cneed = xb.xnor_conv2d_chain_workspace_bytes(s)
    assert cneed > need
    assert L.xnor_conv2d_fwd_chain(ok, ok, ok, None, ok, sp, None, ok, ok, cneed, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd_chain(ok, ok, ok, None, ok, sp, ok, ok, None, cneed, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd_chain(ok, ok, None, None, ok, sp, ok, ok, ok, cneed, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd_chain(ok, ok, ok, ok, ok, sp, ok, ok, ok, cneed, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd_chain(ok, ok, ok, None, ok, sp, ok, ok, ok, cneed - 1, None) == xb.E_WORKSPACE
    assert L.xnor_conv2d_fwd_chain(ok, ok, ok, None, ok, sp, odd, ok, ok, cneed, None) == xb.E_ALIGN
    assert L.xnor_conv2d_fwd_chain(ok, ok, None, odd, ok, sp, ok, ok, ok, cneed, None) == xb.E_ALIGN
    assert L.xnor_conv2d_fwd_chain(ok, odd, None, ok, ok, sp, ok, ok, ok, cneed, None) == xb.E_ALIGN
    # (no Wpk: the filters are already expanded in the workspace)
    assert L.xnor_conv2d_fwd_chain(ok, None, None, ok, ok, sp, ok, ok, None, cneed, None) == xb.E_NULL
    assert L.xnor_conv2d_fwd_chain(ok, None, None, ok, ok, sp, ok, ok, ok, cneed - 1, None) == xb.E_WORKSPACE
    assert L.xnor_conv2d_fwd_chain(ok, None, None, odd, ok, sp, ok, ok, ok, cneed, None) == xb.E_ALIGN
    assert L.xnor_box_filter_K(None, sp, ok, None) == xb.E_NULL
    assert L.xnor_box_filter_K(ok, sp, odd, None) == xb.E_ALIGN
    # the one-kernel pass for few-channel images: this 64-channel shape is not its business
    assert not xb.xnor_forward_image_supported(s)
    assert L.xnor_forward_image(ok, ok, ok, sp, ok, None, None) == xb.E_UNSUPPORTED
    img = xb.Shape(1, 1, 256, 256, 1, 3, 3, 1, 1, 1, 1)
    ip = ctypes.byref(img.c())
    assert xb.xnor_forward_image_supported(img)
    assert xb.xnor_forward_image_supported(xb.Shape(2, 4, 30, 30, 9, 7, 7, 1, 1, 0, 0))
    assert xb.xnor_forward_image_supported(xb.Shape(1, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3))
    assert not xb.xnor_forward_image_supported(xb.Shape(1, 1, 256, 256, 1, 3, 5, 1, 1, 1, 2))
    assert L.xnor_forward_image(None, ok, ok, ip, ok, None, None) == xb.E_NULL
    assert L.xnor_forward_image(ok, ok, ok, ip, None, None, None) == xb.E_NULL
    assert L.xnor_forward_image(ok, ok, ok, ip, odd, None, None) == xb.E_ALIGN
    assert L.xnor_forward_image(ok, ok, ok, ip, ok, odd, None) == xb.E_ALIGN
    assert L.xnor_forward_image_supported(None) == xb.E_NULL
    # Binary-Weight-Network layer
    assert L.xnor_bwn_conv2d_fwd(None, ok, ok, sp, ok, None) == xb.E_NULL
    assert L.xnor_bwn_conv2d_fwd(ok, ok, ok, sp, None, None) == xb.E_NULL
    assert L.xnor_bwn_conv2d_fwd(ok, odd, ok, sp, ok, None) == xb.E_ALIGN
    assert L.xnor_bwn_conv2d_fwd_algo(ok, ok, ok, sp, ok, xb.ALGO_TILED, None) == xb.E_UNSUPPORTED
    assert L.xnor_bwn_conv2d_fwd_algo(ok, ok, ok, sp, ok, 99, None) == xb.E_UNSUPPORTED
    wide = xb.Shape(1, 64, 8, 4000, 8, 3, 3, 1, 1, 1, 1)      # rows too wide for the matrix-core kernel's LDS band
    assert L.xnor_bwn_conv2d_fwd_algo(ok, ok, ok, ctypes.byref(wide.c()), ok, xb.ALGO_MFMA, None) == xb.E_UNSUPPORTED
    # the three-term bf16 kernel: up to 64 taps, and rows that fit its staging
    assert L.xnor_bwn_conv2d_fwd_algo(ok, ok, ok, ctypes.byref(wide.c()), ok, xb.ALGO_MFMA_SPLIT, None) == xb.E_UNSUPPORTED
    nine = xb.Shape(1, 64, 16, 16, 8, 9, 9, 1, 1, 4, 4)
    assert L.xnor_bwn_conv2d_fwd_algo(ok, ok, ok, ctypes.byref(nine.c()), ok, xb.ALGO_MFMA_SPLIT, None) == xb.E_UNSUPPORTED
    assert L.xnor_bwn_conv2d_fwd_algo(None, ok, ok, sp, ok, xb.ALGO_MFMA_SPLIT, None) == xb.E_NULL


def _rows_spanned(OH, OW, tiles, row_segments):
    """Most output rows any workgroup's tiles touch, by walking every workgroup's tiles."""
    worst = 0
    if row_segments:
        total = OH * row_segments
        for t0 in range(0, total, tiles):
            t1 = min(total, t0 + tiles)
            worst = max(worst, (t1 - 1) // row_segments - t0 // row_segments + 1)
    else:
        total = (OH * OW + 31) // 32
        for t0 in range(0, total, tiles):
            last = min(OH * OW, min(total, t0 + tiles) * 32) - 1
            worst = max(worst, last // OW - (t0 * 32) // OW + 1)
    return worst, total


def test_bwn_split_plan_holds_what_its_tiles_need(xb):
    """The launch plan of the three-term bf16 kernel, on the benchmark layers and on seeded random
    shapes, for several unit counts: the staged positions it sizes the LDS for cover the input rows
    under the output rows that any workgroup's tiles really touch (walked tile by tile here), within
    the kernel's limits, and the grid is N x filter groups x tile groups."""
    import numpy as np
    from paper_2007_14178_amd.workloads import LAYERS
    shapes = [(L.N, L.C, L.H, L.W, L.F, L.kh, L.kw, L.sh, L.sw, L.ph, L.pw) for L in LAYERS.values()]
    rng = np.random.default_rng(77)
    for _ in range(300):
        kh, kw = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        H, W = int(rng.integers(kh, 90)), int(rng.integers(kw, 140))
        shapes.append((int(rng.integers(1, 20)), int(rng.integers(1, 200)), H, W, int(rng.integers(1, 400)),
                       kh, kw, int(rng.integers(1, 4)), int(rng.integers(1, 4)),
                       int(rng.integers(0, kh)), int(rng.integers(0, kw))))
    seen_modes = set()
    for full in shapes:
        s = xb.Shape(*full)
        N, C, H, W, F, kh, kw, sh, sw, ph, pw = full
        OH, OW = (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1
        for cus in (256, 64, 1):
            try:
                pl = xb.xnor_bwn_split_plan(s, cus)
            except xb.XnorError as e:
                assert e.status == xb.E_UNSUPPORTED, full
                assert xb.xnor_bwn_pick_algo(s) != xb.ALGO_MFMA_SPLIT
                continue
            assert xb.xnor_bwn_pick_algo(s) == xb.ALGO_MFMA_SPLIT
            T, seg, lds = pl["tiles"], pl["row_segments"], pl["lds_bytes"]
            assert 1 <= T <= 6 and lds <= 160 * 1024, (full, pl)
            assert seg in (0, (OW + 31) // 32), (full, pl)
            seen_modes.add(bool(seg))
            body = lds // 2 - 1024 - kh * kw * 128 * 4       # per tile buffer: positions x 112 bytes
            assert lds % 2 == 0 and body > 0 and body % 112 == 0, (full, pl)
            npos = body // 112
            assert npos <= 512, (full, pl)
            rows_out, total = _rows_spanned(OH, OW, T, seg)
            need = ((rows_out - 1) * sh + kh) * (W + 2 * pw)
            assert npos >= need, (full, pl, rows_out)
            assert pl["workgroups"] == N * ((F + 127) // 128) * ((total + T - 1) // T), (full, pl)
    assert seen_modes == {False, True}
    # the two measured cases that motivated the row segments: 56 x 56 outputs, 16 images, 128 filters
    k7 = xb.xnor_bwn_split_plan(xb.Shape(16, 128, 56, 56, 128, 7, 7, 1, 1, 3, 3), 256)
    assert k7["row_segments"] == 2 and k7["tiles"] == 4
    with pytest.raises(xb.XnorError):
        xb.xnor_bwn_split_plan(xb.Shape(1, 64, 8, 4000, 8, 3, 3, 1, 1, 1, 1), 256)
    assert xb.lib.xnor_bwn_split_plan(None, 0, None, None, None, None) == xb.E_NULL
    assert xb.lib.xnor_bwn_pick_algo(None) == xb.E_NULL


def test_probe_arguments_rejected(xb):
    """The measurement probes check their arguments before any HIP call."""
    L = xb.lib
    ok = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    x = ctypes.c_double()
    assert L.xnor_probe_mfma_fp4(256, 10, None, ctypes.byref(x), None) == xb.E_NULL
    assert L.xnor_probe_mfma_fp4(0, 10, ok, ctypes.byref(x), None) == xb.E_SHAPE
    assert L.xnor_probe_mfma_fp4(256, 0, ok, ctypes.byref(x), None) == xb.E_SHAPE
    assert L.xnor_probe_mfma_bf16(256, 10, 1, ok, None, None) == xb.E_NULL
    assert L.xnor_probe_mfma_bf16((1 << 20) + 1, 10, 0, ok, ctypes.byref(x), None) == xb.E_SHAPE
    assert L.xnor_probe_xor_popcount(256, (1 << 24) + 1, ok, ctypes.byref(x), None) == xb.E_SHAPE
    assert L.xnor_probe_copy(None, ok, 1024, None) == xb.E_NULL
    assert L.xnor_probe_copy(ok, ok, 1000, None) == xb.E_SHAPE
    assert L.xnor_probe_copy(ok, odd, 1024, None) == xb.E_ALIGN
    assert L.xnor_probe_read(ok, 0, ok, None) == xb.E_SHAPE
    assert L.xnor_probe_read(odd, 1024, ok, None) == xb.E_ALIGN
    assert L.xnor_probe_read(ok, 1024, None, None) == xb.E_NULL
    big = 256 * 8 * 131072
    assert L.xnor_probe_store_beside_mfma(256, 8, 1, 1, None, big, ok, ok, None) == xb.E_NULL
    assert L.xnor_probe_store_beside_mfma(256, 8, 1, 1, ok, big - 1, ok, ok, None) == xb.E_SHAPE     # dst too small
    assert L.xnor_probe_store_beside_mfma(256, 65, 1, 1, ok, 256 * 65 * 131072, ok, ok, None) == xb.E_SHAPE
    assert L.xnor_probe_store_beside_mfma(4097, 1, 1, 1, ok, 4097 * 131072, ok, ok, None) == xb.E_SHAPE
    assert L.xnor_probe_store_beside_mfma(256, 8, 0, 3, ok, big, ok, ok, None) == xb.E_SHAPE
    assert L.xnor_probe_store_beside_mfma(256, 8, 0, 0, odd, big, ok, ok, None) == xb.E_ALIGN


def test_binding_refuses_cpu_tensors(xb):
    import torch
    with pytest.raises(TypeError):
        xb.xnor_binarize_pack(torch.zeros(1, 32, 2, 2))
    with pytest.raises(TypeError):
        xb.xnor_alpha(torch.zeros(2, 32, 3, 3))


def test_workloads_are_seeded_and_shaped():
    import numpy as np
    from paper_2007_14178_amd.workloads import LAYERS, make_input, make_weights
    L = LAYERS["c5"]
    assert (L.OH, L.OW, L.n_red, L.binary_macs) == (28, 28, 4608, 128 * 512 * 784 * 4608)
    a, b = make_input(L, 2), make_input(L, 1)
    assert a.shape == (2, 512, 28, 28) and a.dtype == np.float32 and np.array_equal(a[:1], b)
    assert 0.04 < (a == 0).mean() < 0.06
    w = make_weights(LAYERS["c3_s1"])
    assert w.shape == (256, 256, 3, 3) and abs(w.std() - 0.05) < 0.002
    u = make_input(LAYERS["c4_conv3"], 1)
    assert u.min() >= -1 and u.max() <= 1 and abs(u.mean()) < 0.01
    assert LAYERS["c3_s2"].OH == 14 and LAYERS["c4_conv2"].OH == 27 and LAYERS["c2_k7"].n_red == 6272
