"""Chained layers: xnor_conv2d_fwd_chain and xnor_box_filter_K against the oracle.

What the chained call must produce is what the next layer's input stage would compute from this
layer's fp32 output O, so the expected values are compositions of oracle functions that are pinned
on their own: Opk = pack(O_ref) bit for bit, A_next = channel_mean_abs(O_ref) within 1e-5.  The last
test runs two layers back to back on the GPU without ever forming an fp32 tensor in between and
compares with the oracle run layer by layer.
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


def assert_rel(got, ref, what, rtol=RTOL):
    got = got.astype(np.float64); ref = ref.astype(np.float64)
    err = np.abs(got - ref)
    bad = err > np.maximum(rtol * np.abs(ref), 2.0 ** -149)   # (one subnormal spacing where that is larger)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside {rtol} rel; worst {err.max()}"


#        N   C   H   W   F  kh kw sh sw ph pw
SHAPES = [
    (1, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1),
    (2, 32, 13, 13, 33, 3, 3, 1, 1, 1, 1),       # F = 33: a word with one live bit
    (3, 65, 12, 20, 9, 3, 5, 2, 1, 1, 2),        # F < 32, strides, channel tail
    (2, 96, 27, 27, 200, 5, 5, 1, 1, 2, 2),      # two filter tiles, the second partly empty
    (5, 256, 14, 14, 130, 3, 3, 1, 1, 1, 1),     # bands that run across images
    (1, 512, 28, 28, 96, 3, 3, 1, 1, 1, 1),      # several channel chunks
    (2, 40, 9, 9, 4, 3, 3, 1, 1, 3, 2),          # windows that are all padding: K = 0 there
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_chain_outputs_vs_oracle(xb, shape):
    print(f"case chain shape={shape}", flush=True)
    rng = np.random.default_rng(zlib.crc32(("chain" + str(shape)).encode()))
    layer, I, Wt = random_layer(rng, "t", *shape)
    s = xb.Shape(*shape)
    osh = oracle.Shape(*shape)
    Ipk, K, A = xb.xnor_input_prepare(dev(I), s)
    Wpk, alpha, _ = xb.xnor_filter_prepare(dev(Wt))
    Opk, A_next = xb.xnor_conv2d_fwd_chain(Ipk, Wpk, K, alpha, s)
    # the form that takes the channel mean and forms K itself gives the same bits
    Opk2, A_next2 = xb.xnor_conv2d_fwd_chain(Ipk, Wpk, None, alpha, s, A=A)
    # ... and so does the form whose filters were expanded beforehand, into the chain workspace
    cws = torch.empty((xb.xnor_conv2d_chain_workspace_bytes(s),), dtype=torch.uint8, device="cuda")
    xb.xnor_filter_expand(Wpk, s, cws)
    Opk3, A_next3 = xb.xnor_conv2d_fwd_chain(Ipk, None, None, alpha, s, workspace=cws, A=A)
    Opk4, A_next4 = xb.xnor_conv2d_fwd_chain(Ipk, None, None, alpha, s, workspace=cws, A=A)   # (the filters are only read)
    torch.cuda.synchronize()
    assert torch.equal(Opk, Opk2) and torch.equal(A_next, A_next2)
    assert torch.equal(Opk, Opk3) and torch.equal(A_next, A_next3)
    assert torch.equal(Opk, Opk4) and torch.equal(A_next, A_next4)
    d_ref, K_ref, a_ref, O_ref = oracle.forward(I, Wt, osh)
    assert np.array_equal(Opk.cpu().numpy().view(np.uint32), oracle.pack(O_ref)), "packed signs of the output"
    A_ref = oracle.channel_mean_abs(O_ref)
    got = A_next.cpu().numpy()
    assert_rel(got, A_ref, "channel mean of |out|")
    assert np.array_equal(got == 0, A_ref == 0)


@pytest.mark.parametrize("name", ["c1", "c3_s2", "c4_conv3", "c5"])
def test_chain_benchmark_layers_reduced_batch(xb, name):
    full = LAYERS[name]
    n = 1 if full.binary_macs // full.N > 1.5e9 else min(full.N, 2)
    layer = full.with_batch(n)
    print(f"case chain layer={name} N={n}", flush=True)
    I, Wt = make_input(full, n), make_weights(full)
    s = xb.Shape(layer.N, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw, layer.sh, layer.sw, layer.ph, layer.pw)
    osh = oracle.Shape(layer.N, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw, layer.sh, layer.sw, layer.ph, layer.pw)
    Ipk, K, _ = xb.xnor_input_prepare(dev(I), s)
    Wpk, alpha, _ = xb.xnor_filter_prepare(dev(Wt))
    Opk, A_next = xb.xnor_conv2d_fwd_chain(Ipk, Wpk, K, alpha, s)
    torch.cuda.synchronize()
    _, _, _, O_ref = oracle.forward(I, Wt, osh)
    assert np.array_equal(Opk.cpu().numpy().view(np.uint32), oracle.pack(O_ref))
    assert_rel(A_next.cpu().numpy(), oracle.channel_mean_abs(O_ref), "channel mean of |out|")


@pytest.mark.parametrize("geom", [(3, 17, 9, 3, 3, 1, 1, 1, 1), (2, 28, 28, 5, 5, 2, 2, 2, 2), (1, 6, 40, 1, 3, 1, 2, 0, 1)])
def test_box_filter_K_vs_oracle(xb, geom):
    """K from a given A.  With one input channel the oracle's A is |I| exactly, so its K is the box
    filter of a known A."""
    N, H, W, kh, kw, sh, sw, ph, pw = geom
    rng = np.random.default_rng(zlib.crc32(("box" + str(geom)).encode()))
    A = np.abs(rng.standard_normal((N, H, W)).astype(np.float32))
    s = xb.Shape(N, 1, H, W, 1, kh, kw, sh, sw, ph, pw)
    K = xb.xnor_box_filter_K(dev(A), s)
    torch.cuda.synchronize()
    K_ref = oracle.scale_K(A[:, None], oracle.Shape(N, 1, H, W, 1, kh, kw, sh, sw, ph, pw))
    assert_rel(K.cpu().numpy(), K_ref, "K")


def test_two_chained_layers(xb):
    """Layer 1 -> (packed signs, A) -> layer 2, no fp32 activation in between, against the oracle run
    layer by layer.  The packed hand-over must be bit-exact; layer 2's K comes from a channel mean
    that is itself within 1e-5, so K2 and the final output are held to 3e-5."""
    rng = np.random.default_rng(77)
    s1 = (2, 64, 20, 20, 96, 3, 3, 1, 1, 1, 1)
    _, I, W1 = random_layer(rng, "l1", *s1)
    s2 = (2, 96, 20, 20, 40, 3, 3, 2, 2, 1, 1)
    _, _, W2 = random_layer(rng, "l2", *s2)
    S1, S2 = xb.Shape(*s1), xb.Shape(*s2)
    Ipk, K1, _ = xb.xnor_input_prepare(dev(I), S1)
    W1pk, a1, _ = xb.xnor_filter_prepare(dev(W1))
    W2pk, a2, _ = xb.xnor_filter_prepare(dev(W2))
    O1pk, A2 = xb.xnor_conv2d_fwd_chain(Ipk, W1pk, K1, a1, S1)
    K2 = xb.xnor_box_filter_K(A2, S2)
    out2, dot2 = xb.xnor_conv2d_fwd(O1pk, W2pk, K2, a2, S2, want_dot=True)
    torch.cuda.synchronize()
    _, _, _, O1_ref = oracle.forward(I, W1, oracle.Shape(*s1))
    d2_ref, K2_ref, _, O2_ref = oracle.forward(O1_ref, W2, oracle.Shape(*s2))
    assert np.array_equal(O1pk.cpu().numpy().view(np.uint32), oracle.pack(O1_ref))
    assert np.array_equal(dot2.cpu().numpy(), d2_ref)
    assert_rel(K2.cpu().numpy(), K2_ref, "K of layer 2", rtol=3e-5)
    assert_rel(out2.cpu().numpy(), O2_ref, "output of layer 2", rtol=3e-5)
