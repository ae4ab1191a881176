"""The entry point that allocates nothing (xnor_conv2d_fwd_static: workspace in the library's own
static device array) gives what xnor_conv2d_fwd_algo(XNOR_ALGO_MFMA) gives with a caller's workspace:
dot products bit for bit, outputs within the parity bar of the oracle and identical to the existing
entry point's.  Two calls in a row share the array: the second, on a smaller layer, must not see the
first's contents.  Collected last on purpose (the name), and passes alone in a fresh process too."""
import zlib

import numpy as np
import pytest
import torch

import oracle
from paper_2007_14178_amd.workloads import random_layer

pytestmark = pytest.mark.gpu

RTOL = 1e-5


def run_both(xb, shape, seed_tag):
    rng = np.random.default_rng(zlib.crc32((seed_tag + str(shape)).encode()))
    layer, I, Wt = random_layer(rng, "t", *shape)
    s = xb.Shape(*shape)
    OH, OW = xb.xnor_out_dim(s)
    dI = torch.from_numpy(I).cuda()
    dW = torch.from_numpy(Wt).cuda()
    Ipk, K, A = xb.xnor_input_prepare(dI, s)
    Wpk, alpha, _ = xb.xnor_filter_prepare(dW)
    assert 0 < xb.xnor_conv2d_workspace_bytes(s) <= xb.STATIC_SCRATCH_BYTES
    out = torch.full((s.N, s.F, OH, OW), float("nan"), dtype=torch.float32, device="cuda")
    dot = torch.full((s.N, s.F, OH, OW), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    xb.xnor_conv2d_fwd_static(Ipk, Wpk, K, alpha, s, out, dot)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    out_ref, dot_ref = xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, want_dot=True, algo=xb.ALGO_MFMA)
    torch.cuda.synchronize()
    assert torch.equal(dot, dot_ref), "dot vs the existing entry point"
    assert torch.equal(out, out_ref), "out vs the existing entry point"
    d_o, K_o, a_o, O_o = oracle.forward(I, Wt, oracle.Shape(*shape))
    assert np.array_equal(dot.cpu().numpy(), d_o), "dot vs the oracle"
    got = out.cpu().numpy().astype(np.float64)
    err = np.abs(got - O_o.astype(np.float64))
    floor = (0.5 * np.abs(d_o.astype(np.float64)) * (a_o.astype(np.float64)[None, :, None, None] + 1.0) + 1.0) * 2.0 ** -149
    assert not (err > np.maximum(RTOL * np.abs(O_o), floor)).any(), "out vs the oracle"


def test_static_scratch_two_calls_second_smaller():
    from paper_2007_14178_amd import binding as xb
    print("case static scratch, larger layer", flush=True)
    run_both(xb, (3, 512, 28, 28, 200, 3, 3, 1, 1, 1, 1), "static")     # several chunks, ragged filter tile
    print("case static scratch, smaller layer", flush=True)
    run_both(xb, (2, 96, 14, 14, 40, 3, 3, 1, 1, 1, 1), "static")       # one chunk, fewer filters, smaller layout


def test_static_scratch_rejects_what_does_not_fit():
    from paper_2007_14178_amd import binding as xb
    # filters whose expanded form is beyond the array: rejected before anything is launched
    s = xb.Shape(1, 2048, 14, 14, 1024, 3, 3, 1, 1, 1, 1)
    assert xb.xnor_conv2d_workspace_bytes(s) > xb.STATIC_SCRATCH_BYTES
    OH, OW = xb.xnor_out_dim(s)
    z = lambda shape, dt: torch.zeros(shape, dtype=dt, device="cuda")
    with pytest.raises(xb.XnorError) as e:
        xb.xnor_conv2d_fwd_static(z((s.N, s.H, s.W, s.Cw), torch.int32), z((s.F, s.kh, s.kw, s.Cw), torch.int32),
                                  z((s.N, OH, OW), torch.float32), z((s.F,), torch.float32), s,
                                  z((s.N, s.F, OH, OW), torch.float32))
    assert e.value.status == xb.E_WORKSPACE
