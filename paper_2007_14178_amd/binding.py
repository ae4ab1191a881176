"""ctypes binding of the C ABI in include/xnor.h -- argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks dtype / shape /
contiguity, and passes raw device pointers plus the current HIP stream to the library call of the
same name.  No step of the pipeline runs in Python or in torch: if the HIP library is missing the
import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libxnor_hip.so")

ALGO_AUTO, ALGO_DIRECT, ALGO_TILED, ALGO_MFMA, ALGO_MFMA_BANDS, ALGO_MFMA_SPLIT = 0, 1, 2, 3, 4, 5
ALGO_NAMES = {ALGO_AUTO: "auto", ALGO_DIRECT: "direct", ALGO_TILED: "tiled", ALGO_MFMA: "mfma",
              ALGO_MFMA_BANDS: "mfma_bands", ALGO_MFMA_SPLIT: "mfma_split"}
E_NULL, E_SHAPE, E_ALIGN, E_HIP, E_UNSUPPORTED, E_WORKSPACE = -1, -2, -3, -4, -5, -6


class XnorError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.xnor_strerror(status).decode()
        if status == E_HIP:
            msg += ": " + lib.xnor_last_hip_error().decode()
        super().__init__(f"{where}: {msg} (status {status})")


class CShape(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in
                ("N", "C", "H", "W", "F", "kh", "kw", "sh", "sw", "ph", "pw")]


@dataclass(frozen=True)
class Shape:
    N: int
    C: int
    H: int
    W: int
    F: int
    kh: int
    kw: int
    sh: int = 1
    sw: int = 1
    ph: int = 0
    pw: int = 0

    def c(self) -> CShape:
        # (built once per Shape: the struct is read-only on the C side)
        cs = self.__dict__.get("_c")
        if cs is None:
            cs = CShape(self.N, self.C, self.H, self.W, self.F, self.kh, self.kw,
                        self.sh, self.sw, self.ph, self.pw)
            object.__setattr__(self, "_c", cs)
        return cs

    @property
    def Cw(self) -> int:
        return (self.C + 31) // 32


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2007_14178_amd.build` "
            "(there is no CPU or PyTorch fallback for the XNOR pipeline)")
    L = ctypes.CDLL(LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    sp = ctypes.POINTER(CShape)
    L.xnor_out_dim.argtypes = [sp, ctypes.POINTER(ci), ctypes.POINTER(ci)]
    L.xnor_packed_words.argtypes = [ci]
    L.xnor_strerror.argtypes = [ci]
    L.xnor_strerror.restype = ctypes.c_char_p
    L.xnor_last_hip_error.argtypes = []
    L.xnor_last_hip_error.restype = ctypes.c_char_p
    L.xnor_binarize_pack.argtypes = [vp, ci, ci, ci, ci, vp, vp]
    L.xnor_scale_K.argtypes = [vp, sp, vp, vp, vp]
    L.xnor_alpha.argtypes = [vp, ci, ci, ci, ci, vp, vp]
    L.xnor_input_prepare.argtypes = [vp, sp, vp, vp, vp, vp]
    L.xnor_filter_prepare.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp]
    sz = ctypes.c_size_t
    L.xnor_prepare.argtypes = [vp, vp, sp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.xnor_conv2d_fwd.argtypes = [vp, vp, vp, vp, sp, vp, vp, vp, sz, vp]
    L.xnor_conv2d_fwd_algo.argtypes = [vp, vp, vp, vp, sp, vp, vp, vp, sz, ci, vp]
    L.xnor_conv2d_fwd_static.argtypes = [vp, vp, vp, vp, sp, vp, vp, vp]
    L.xnor_filter_expand.argtypes = [vp, sp, vp, sz, vp]
    dp = ctypes.POINTER(ctypes.c_double)
    L.xnor_probe_mfma_fp4.argtypes = [ci, ci, vp, dp, vp]
    L.xnor_probe_mfma_bf16.argtypes = [ci, ci, ci, vp, dp, vp]
    L.xnor_probe_xor_popcount.argtypes = [ci, ci, vp, dp, vp]
    L.xnor_probe_copy.argtypes = [vp, vp, sz, vp]
    L.xnor_probe_read.argtypes = [vp, sz, vp, vp]
    L.xnor_probe_store_beside_mfma.argtypes = [ci, ci, ci, ci, vp, sz, vp, vp, vp]
    L.xnor_conv2d_fwd_expanded.argtypes = [vp, vp, sz, vp, vp, vp, sp, vp, vp, vp]
    L.xnor_box_filter_K.argtypes = [vp, sp, vp, vp]
    L.xnor_conv2d_chain_workspace_bytes.argtypes = [sp, ctypes.POINTER(sz)]
    L.xnor_conv2d_fwd_chain.argtypes = [vp, vp, vp, vp, vp, sp, vp, vp, vp, sz, vp]
    L.xnor_forward_image_supported.argtypes = [sp]
    L.xnor_forward_image.argtypes = [vp, vp, vp, sp, vp, vp, vp]
    L.xnor_bwn_conv2d_fwd.argtypes = [vp, vp, vp, sp, vp, vp]
    L.xnor_bwn_conv2d_fwd_algo.argtypes = [vp, vp, vp, sp, vp, ci, vp]
    L.xnor_conv2d_fp32_fwd.argtypes = [vp, vp, sp, vp, vp]
    L.xnor_conv2d_fp32_fwd_algo.argtypes = [vp, vp, sp, vp, ci, vp]
    L.xnor_conv2d_pick_algo.argtypes = [sp, sz]
    L.xnor_bwn_pick_algo.argtypes = [sp]
    L.xnor_bwn_split_plan.argtypes = [sp, ci, ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(sz),
                                      ctypes.POINTER(ctypes.c_longlong)]
    L.xnor_conv2d_workspace_bytes.argtypes = [sp, ctypes.POINTER(sz)]
    for name in ("xnor_out_dim", "xnor_packed_words", "xnor_binarize_pack", "xnor_scale_K",
                 "xnor_alpha", "xnor_conv2d_fwd", "xnor_conv2d_fwd_algo", "xnor_conv2d_pick_algo",
                 "xnor_conv2d_workspace_bytes", "xnor_input_prepare", "xnor_filter_prepare",
                 "xnor_filter_expand", "xnor_conv2d_fwd_expanded", "xnor_box_filter_K",
                 "xnor_conv2d_chain_workspace_bytes", "xnor_conv2d_fwd_chain",
                 "xnor_forward_image_supported", "xnor_forward_image",
                 "xnor_bwn_conv2d_fwd", "xnor_bwn_conv2d_fwd_algo",
                 "xnor_prepare", "xnor_conv2d_fwd_static",
                 "xnor_probe_mfma_fp4", "xnor_probe_mfma_bf16", "xnor_probe_xor_popcount", "xnor_probe_copy", "xnor_probe_read",
                 "xnor_conv2d_fp32_fwd", "xnor_conv2d_fp32_fwd_algo"):
        getattr(L, name).restype = ci
    return L


lib = _load()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, shape=None, name="tensor") -> int:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: need a contiguous {dtype} GPU tensor, got {t.dtype} on {t.device}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)} != expected {tuple(shape)}")
    return t.data_ptr()


def _ok(status: int, where: str):
    if status != 0:
        raise XnorError(status, where)


def xnor_out_dim(s: Shape) -> tuple[int, int]:
    dims = s.__dict__.get("_out_dim")       # asked on every call: remembered per Shape
    if dims is None:
        oh, ow = ctypes.c_int(), ctypes.c_int()
        _ok(lib.xnor_out_dim(ctypes.byref(s.c()), ctypes.byref(oh), ctypes.byref(ow)), "xnor_out_dim")
        dims = (oh.value, ow.value)
        object.__setattr__(s, "_out_dim", dims)
    return dims


def xnor_packed_words(C: int) -> int:
    r = lib.xnor_packed_words(C)
    if r < 0:
        raise XnorError(r, "xnor_packed_words")
    return r


def xnor_binarize_pack(x: torch.Tensor, packed: torch.Tensor | None = None) -> torch.Tensor:
    """x fp32 [N][C][H][W] -> int32-typed tensor of uint32 words [N][H][W][ceil(C/32)]."""
    N, C, H, W = x.shape
    if packed is None:
        packed = torch.empty((N, H, W, (C + 31) // 32), dtype=torch.int32, device=x.device)
    _ok(lib.xnor_binarize_pack(_dev(x, torch.float32, name="x"), N, C, H, W,
                               _dev(packed, torch.int32, (N, H, W, (C + 31) // 32), "packed"),
                               _stream()), "xnor_binarize_pack")
    return packed


def xnor_scale_K(I: torch.Tensor, s: Shape, A_work: torch.Tensor | None = None,
                 K: torch.Tensor | None = None) -> tuple[torch.Tensor, torch.Tensor]:
    """Returns (K [N][OH][OW], A [N][H][W])."""
    OH, OW = xnor_out_dim(s)
    if A_work is None:
        A_work = torch.empty((s.N, s.H, s.W), dtype=torch.float32, device=I.device)
    if K is None:
        K = torch.empty((s.N, OH, OW), dtype=torch.float32, device=I.device)
    _ok(lib.xnor_scale_K(_dev(I, torch.float32, (s.N, s.C, s.H, s.W), "I"), ctypes.byref(s.c()),
                         _dev(A_work, torch.float32, (s.N, s.H, s.W), "A_work"),
                         _dev(K, torch.float32, (s.N, OH, OW), "K"), _stream()), "xnor_scale_K")
    return K, A_work


def xnor_alpha(Wt: torch.Tensor, alpha: torch.Tensor | None = None) -> torch.Tensor:
    F, C, kh, kw = Wt.shape
    if alpha is None:
        alpha = torch.empty((F,), dtype=torch.float32, device=Wt.device)
    _ok(lib.xnor_alpha(_dev(Wt, torch.float32, name="Wt"), F, C, kh, kw,
                       _dev(alpha, torch.float32, (F,), "alpha"), _stream()), "xnor_alpha")
    return alpha


def xnor_input_prepare(I: torch.Tensor, s: Shape, Ipk: torch.Tensor | None = None,
                       A_work: torch.Tensor | None = None, K: torch.Tensor | None = None, want_K: bool = True):
    """One pass over I: returns (Ipk, K, A); with want_K=False K is not computed (returned as None)."""
    OH, OW = xnor_out_dim(s)
    if Ipk is None:
        Ipk = torch.empty((s.N, s.H, s.W, s.Cw), dtype=torch.int32, device=I.device)
    if A_work is None:
        A_work = torch.empty((s.N, s.H, s.W), dtype=torch.float32, device=I.device)
    if K is None and want_K:
        K = torch.empty((s.N, OH, OW), dtype=torch.float32, device=I.device)
    _ok(lib.xnor_input_prepare(_dev(I, torch.float32, (s.N, s.C, s.H, s.W), "I"), ctypes.byref(s.c()),
                               _dev(Ipk, torch.int32, (s.N, s.H, s.W, s.Cw), "Ipk"),
                               _dev(A_work, torch.float32, (s.N, s.H, s.W), "A_work"),
                               _dev(K, torch.float32, (s.N, OH, OW), "K") if want_K else None, _stream()),
        "xnor_input_prepare")
    return Ipk, K, A_work


def xnor_prepare(I: torch.Tensor, Wt: torch.Tensor, s: Shape, Ipk: torch.Tensor | None = None,
                 A_work: torch.Tensor | None = None, K: torch.Tensor | None = None, Wpk: torch.Tensor | None = None,
                 M_work: torch.Tensor | None = None, alpha: torch.Tensor | None = None, want_K: bool = True,
                 workspace: torch.Tensor | None = None):
    """Input side and filter side in one call: returns (Ipk, K or None, A, Wpk, alpha, M).
    With ``workspace`` (uint8, xnor_conv2d_workspace_bytes) the expanded filters are left in it."""
    OH, OW = xnor_out_dim(s)
    dev = I.device
    if Ipk is None:
        Ipk = torch.empty((s.N, s.H, s.W, s.Cw), dtype=torch.int32, device=dev)
    if A_work is None:
        A_work = torch.empty((s.N, s.H, s.W), dtype=torch.float32, device=dev)
    if K is None and want_K:
        K = torch.empty((s.N, OH, OW), dtype=torch.float32, device=dev)
    if Wpk is None:
        Wpk = torch.empty((s.F, s.kh, s.kw, s.Cw), dtype=torch.int32, device=dev)
    if M_work is None:
        M_work = torch.empty((s.F, s.kh, s.kw), dtype=torch.float32, device=dev)
    if alpha is None:
        alpha = torch.empty((s.F,), dtype=torch.float32, device=dev)
    _ok(lib.xnor_prepare(_dev(I, torch.float32, (s.N, s.C, s.H, s.W), "I"), _dev(Wt, torch.float32, (s.F, s.C, s.kh, s.kw), "Wt"),
                         ctypes.byref(s.c()), _dev(Ipk, torch.int32, (s.N, s.H, s.W, s.Cw), "Ipk"),
                         _dev(A_work, torch.float32, (s.N, s.H, s.W), "A_work"),
                         _dev(K, torch.float32, (s.N, OH, OW), "K") if want_K else None,
                         _dev(Wpk, torch.int32, (s.F, s.kh, s.kw, s.Cw), "Wpk"),
                         _dev(M_work, torch.float32, (s.F, s.kh, s.kw), "M_work"),
                         _dev(alpha, torch.float32, (s.F,), "alpha"),
                         _dev(workspace, torch.uint8, name="workspace") if workspace is not None else None,
                         workspace.numel() if workspace is not None else 0, _stream()), "xnor_prepare")
    return Ipk, (K if want_K else None), A_work, Wpk, alpha, M_work


def xnor_filter_prepare(Wt: torch.Tensor, Wpk: torch.Tensor | None = None,
                        M_work: torch.Tensor | None = None, alpha: torch.Tensor | None = None):
    """One pass over Wt: returns (Wpk, alpha, M) with M = mean_c |Wt| per tap."""
    F, C, kh, kw = Wt.shape
    Cw = (C + 31) // 32
    if Wpk is None:
        Wpk = torch.empty((F, kh, kw, Cw), dtype=torch.int32, device=Wt.device)
    if M_work is None:
        M_work = torch.empty((F, kh, kw), dtype=torch.float32, device=Wt.device)
    if alpha is None:
        alpha = torch.empty((F,), dtype=torch.float32, device=Wt.device)
    _ok(lib.xnor_filter_prepare(_dev(Wt, torch.float32, name="Wt"), F, C, kh, kw,
                                _dev(Wpk, torch.int32, (F, kh, kw, Cw), "Wpk"),
                                _dev(M_work, torch.float32, (F, kh, kw), "M_work"),
                                _dev(alpha, torch.float32, (F,), "alpha"), _stream()), "xnor_filter_prepare")
    return Wpk, alpha, M_work


def xnor_conv2d_workspace_bytes(s: Shape) -> int:
    n = ctypes.c_size_t()
    _ok(lib.xnor_conv2d_workspace_bytes(ctypes.byref(s.c()), ctypes.byref(n)), "xnor_conv2d_workspace_bytes")
    return n.value


def xnor_conv2d_pick_algo(s: Shape, workspace_bytes: int = 0) -> int:
    r = lib.xnor_conv2d_pick_algo(ctypes.byref(s.c()), workspace_bytes)
    if r < 0:
        raise XnorError(r, "xnor_conv2d_pick_algo")
    return r


def xnor_conv2d_fwd(Ipk: torch.Tensor, Wpk: torch.Tensor, K: torch.Tensor, alpha: torch.Tensor,
                    s: Shape, out: torch.Tensor | None = None, dot: torch.Tensor | None = None,
                    want_dot: bool = False, algo: int = ALGO_AUTO,
                    workspace: torch.Tensor | None | str = "auto"):
    """Returns (out fp32 [N][F][OH][OW], dot int32 or None).

    ``workspace``: a uint8 GPU tensor, None (run a kernel that needs none), or "auto" (allocate what
    xnor_conv2d_workspace_bytes asks for -- callers in a timed loop pass their own buffer)."""
    OH, OW = xnor_out_dim(s)
    oshape = (s.N, s.F, OH, OW)
    if out is None:
        out = torch.empty(oshape, dtype=torch.float32, device=Ipk.device)
    if dot is None and want_dot:
        dot = torch.empty(oshape, dtype=torch.int32, device=Ipk.device)
    if isinstance(workspace, str):
        nbytes = xnor_conv2d_workspace_bytes(s)
        workspace = torch.empty((nbytes,), dtype=torch.uint8, device=Ipk.device) if nbytes else None
    ws_ptr = _dev(workspace, torch.uint8, name="workspace") if workspace is not None else None
    ws_bytes = workspace.numel() if workspace is not None else 0
    _ok(lib.xnor_conv2d_fwd_algo(
        _dev(Ipk, torch.int32, (s.N, s.H, s.W, s.Cw), "Ipk"),
        _dev(Wpk, torch.int32, (s.F, s.kh, s.kw, s.Cw), "Wpk"),
        _dev(K, torch.float32, (s.N, OH, OW), "K"), _dev(alpha, torch.float32, (s.F,), "alpha"),
        ctypes.byref(s.c()), _dev(out, torch.float32, oshape, "out"),
        _dev(dot, torch.int32, oshape, "dot") if dot is not None else None,
        ws_ptr, ws_bytes, algo, _stream()), f"xnor_conv2d_fwd[{ALGO_NAMES.get(algo, algo)}]")
    return out, dot


STATIC_SCRATCH_BYTES = 4 << 20


def xnor_conv2d_fwd_static(Ipk: torch.Tensor, Wpk: torch.Tensor, K: torch.Tensor, alpha: torch.Tensor,
                           s: Shape, out: torch.Tensor, dot: torch.Tensor | None = None):
    """The matrix-core convolution with its workspace in the library's own static array: neither
    the call nor this wrapper allocates, so the caller brings ``out`` (and ``dot`` if wanted)."""
    OH, OW = xnor_out_dim(s)
    oshape = (s.N, s.F, OH, OW)
    _ok(lib.xnor_conv2d_fwd_static(
        _dev(Ipk, torch.int32, (s.N, s.H, s.W, s.Cw), "Ipk"),
        _dev(Wpk, torch.int32, (s.F, s.kh, s.kw, s.Cw), "Wpk"),
        _dev(K, torch.float32, (s.N, OH, OW), "K"), _dev(alpha, torch.float32, (s.F,), "alpha"),
        ctypes.byref(s.c()), _dev(out, torch.float32, oshape, "out"),
        _dev(dot, torch.int32, oshape, "dot") if dot is not None else None, _stream()),
        "xnor_conv2d_fwd_static")
    return out, dot


def xnor_probe_mfma_fp4(workgroups: int, iters: int, sink: torch.Tensor) -> float:
    """Enqueues the register-only FP4 matrix-instruction loop; returns the flops it issues."""
    n = ctypes.c_double(0.0)
    _ok(lib.xnor_probe_mfma_fp4(workgroups, iters, _dev(sink, torch.float32, name="sink"), ctypes.byref(n), _stream()),
        "xnor_probe_mfma_fp4")
    return n.value


def xnor_probe_mfma_bf16(workgroups: int, iters: int, random_b: bool, sink: torch.Tensor) -> float:
    """Enqueue the register-only bf16 matrix-instruction loop; returns the flops it issues."""
    n = ctypes.c_double()
    _ok(lib.xnor_probe_mfma_bf16(workgroups, iters, int(bool(random_b)), _dev(sink, torch.float32, name="sink"),
                                 ctypes.byref(n), _stream()), "xnor_probe_mfma_bf16")
    return n.value


def xnor_probe_xor_popcount(workgroups: int, iters: int, sink: torch.Tensor) -> float:
    """Enqueues the register-only v_xor + v_bcnt loop; returns the binary multiply-accumulates it issues."""
    n = ctypes.c_double(0.0)
    _ok(lib.xnor_probe_xor_popcount(workgroups, iters, _dev(sink, torch.int32, name="sink"), ctypes.byref(n), _stream()),
        "xnor_probe_xor_popcount")
    return n.value


def xnor_probe_copy(src: torch.Tensor, dst: torch.Tensor) -> int:
    """Enqueues the plain copy kernel over the whole of ``src``; returns the bytes copied."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("xnor_probe_copy: src and dst differ in size")
    _ok(lib.xnor_probe_copy(_dev(src, src.dtype, name="src"), _dev(dst, dst.dtype, name="dst"), nbytes, _stream()),
        "xnor_probe_copy")
    return nbytes


def xnor_probe_read(src: torch.Tensor, sink: torch.Tensor) -> int:
    """Enqueue a plain 16-byte-per-lane read of `src`; returns the bytes it reads."""
    nbytes = src.numel() * src.element_size()
    _ok(lib.xnor_probe_read(_dev(src, src.dtype, name="src"), nbytes, _dev(sink, torch.int32, name="sink"), _stream()),
        "xnor_probe_read")
    return nbytes


def xnor_probe_store_beside_mfma(workgroups: int, reps: int, wide: bool, matrix_loop: int, dst: torch.Tensor,
                                 cycles: torch.Tensor, sink: torch.Tensor) -> None:
    """Enqueue the store-beside-a-matrix-loop probe; `cycles` (int64 [workgroups][4]) receives the
    storing waves' shader-clock times, `dst` (fp32, workgroups x reps x 128 KB) is written in full."""
    _ok(lib.xnor_probe_store_beside_mfma(workgroups, reps, 1 if wide else 0, matrix_loop,
                                         _dev(dst, torch.float32, name="dst"), dst.numel() * 4,
                                         _dev(cycles, torch.int64, (workgroups, 4), "cycles"),
                                         _dev(sink, torch.float32, name="sink"), _stream()),
        "xnor_probe_store_beside_mfma")


def xnor_filter_expand(Wpk: torch.Tensor, s: Shape, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Per-model half of the matrix-core convolution: fills (and returns) the workspace."""
    if workspace is None:
        workspace = torch.empty((xnor_conv2d_workspace_bytes(s),), dtype=torch.uint8, device=Wpk.device)
    _ok(lib.xnor_filter_expand(_dev(Wpk, torch.int32, (s.F, s.kh, s.kw, s.Cw), "Wpk"), ctypes.byref(s.c()),
                               _dev(workspace, torch.uint8, name="workspace"), workspace.numel(), _stream()),
        "xnor_filter_expand")
    return workspace


def xnor_conv2d_fwd_expanded(Ipk: torch.Tensor, workspace: torch.Tensor, K: torch.Tensor | None, alpha: torch.Tensor,
                             s: Shape, out: torch.Tensor | None = None, dot: torch.Tensor | None = None,
                             want_dot: bool = False, A: torch.Tensor | None = None):
    """Per-input half: the convolution on a workspace filled by xnor_filter_expand for this shape.
    Exactly one of K [N][OH][OW] and A [N][H][W] (K is then formed inside the kernel) is given."""
    OH, OW = xnor_out_dim(s)
    oshape = (s.N, s.F, OH, OW)
    if out is None:
        out = torch.empty(oshape, dtype=torch.float32, device=Ipk.device)
    if dot is None and want_dot:
        dot = torch.empty(oshape, dtype=torch.int32, device=Ipk.device)
    _ok(lib.xnor_conv2d_fwd_expanded(
        _dev(Ipk, torch.int32, (s.N, s.H, s.W, s.Cw), "Ipk"), _dev(workspace, torch.uint8, name="workspace"),
        workspace.numel(), _dev(K, torch.float32, (s.N, OH, OW), "K") if K is not None else None,
        _dev(A, torch.float32, (s.N, s.H, s.W), "A") if A is not None else None,
        _dev(alpha, torch.float32, (s.F,), "alpha"),
        ctypes.byref(s.c()), _dev(out, torch.float32, oshape, "out"),
        _dev(dot, torch.int32, oshape, "dot") if dot is not None else None, _stream()), "xnor_conv2d_fwd_expanded")
    return out, dot


def xnor_forward_image_supported(s: Shape) -> bool:
    rc = lib.xnor_forward_image_supported(ctypes.byref(s.c()))
    if rc < 0:
        _ok(rc, "xnor_forward_image_supported")
    return bool(rc)


def xnor_forward_image(I: torch.Tensor, Wpk: torch.Tensor, alpha: torch.Tensor, s: Shape,
                       out: torch.Tensor | None = None, dot: torch.Tensor | None = None,
                       want_dot: bool = False):
    """Whole forward pass for a few-channel image in one kernel. Returns (out, dot or None)."""
    OH, OW = xnor_out_dim(s)
    oshape = (s.N, s.F, OH, OW)
    if out is None:
        out = torch.empty(oshape, dtype=torch.float32, device=I.device)
    if dot is None and want_dot:
        dot = torch.empty(oshape, dtype=torch.int32, device=I.device)
    _ok(lib.xnor_forward_image(
        _dev(I, torch.float32, (s.N, s.C, s.H, s.W), "I"), _dev(Wpk, torch.int32, (s.F, s.kh, s.kw, s.Cw), "Wpk"),
        _dev(alpha, torch.float32, (s.F,), "alpha"), ctypes.byref(s.c()), _dev(out, torch.float32, oshape, "out"),
        _dev(dot, torch.int32, oshape, "dot") if dot is not None else None, _stream()), "xnor_forward_image")
    return out, dot


def xnor_bwn_pick_algo(s: Shape) -> int:
    r = lib.xnor_bwn_pick_algo(ctypes.byref(s.c()))
    if r < 0:
        raise XnorError(r, "xnor_bwn_pick_algo")
    return r


def xnor_bwn_split_plan(s: Shape, compute_units: int = 0) -> dict:
    """The launch ALGO_MFMA_SPLIT makes for this shape: tiles per workgroup, row segments (0 =
    tiles of consecutive pixels), LDS bytes per workgroup, workgroups."""
    t, r = ctypes.c_int(), ctypes.c_int()
    b, w = ctypes.c_size_t(), ctypes.c_longlong()
    _ok(lib.xnor_bwn_split_plan(ctypes.byref(s.c()), compute_units, ctypes.byref(t), ctypes.byref(r),
                                ctypes.byref(b), ctypes.byref(w)), "xnor_bwn_split_plan")
    return {"tiles": t.value, "row_segments": r.value, "lds_bytes": b.value, "workgroups": w.value}


def xnor_bwn_conv2d_fwd(I: torch.Tensor, Wpk: torch.Tensor, alpha: torch.Tensor, s: Shape,
                        out: torch.Tensor | None = None, algo: int = ALGO_AUTO) -> torch.Tensor:
    """Binary-Weight-Network layer (Eq. 1): real input, packed sign weights, alpha. Returns out."""
    OH, OW = xnor_out_dim(s)
    oshape = (s.N, s.F, OH, OW)
    if out is None:
        out = torch.empty(oshape, dtype=torch.float32, device=I.device)
    _ok(lib.xnor_bwn_conv2d_fwd_algo(
        _dev(I, torch.float32, (s.N, s.C, s.H, s.W), "I"), _dev(Wpk, torch.int32, (s.F, s.kh, s.kw, s.Cw), "Wpk"),
        _dev(alpha, torch.float32, (s.F,), "alpha"), ctypes.byref(s.c()), _dev(out, torch.float32, oshape, "out"),
        algo, _stream()), f"xnor_bwn_conv2d_fwd[{ALGO_NAMES.get(algo, algo)}]")
    return out


def xnor_conv2d_fp32_fwd(I: torch.Tensor, Wt: torch.Tensor, s: Shape, out: torch.Tensor | None = None,
                         algo: int = ALGO_AUTO) -> torch.Tensor:
    """Real-valued convolution (the float comparison of Table I): fp32 input and weights. Returns out."""
    OH, OW = xnor_out_dim(s)
    oshape = (s.N, s.F, OH, OW)
    if out is None:
        out = torch.empty(oshape, dtype=torch.float32, device=I.device)
    _ok(lib.xnor_conv2d_fp32_fwd_algo(
        _dev(I, torch.float32, (s.N, s.C, s.H, s.W), "I"), _dev(Wt, torch.float32, (s.F, s.C, s.kh, s.kw), "Wt"),
        ctypes.byref(s.c()), _dev(out, torch.float32, oshape, "out"), algo, _stream()),
        f"xnor_conv2d_fp32_fwd[{ALGO_NAMES.get(algo, algo)}]")
    return out


def xnor_box_filter_K(A: torch.Tensor, s: Shape, K: torch.Tensor | None = None) -> torch.Tensor:
    """K [N][OH][OW] from a given A [N][H][W] (second half of Eq. 10)."""
    OH, OW = xnor_out_dim(s)
    if K is None:
        K = torch.empty((s.N, OH, OW), dtype=torch.float32, device=A.device)
    _ok(lib.xnor_box_filter_K(_dev(A, torch.float32, (s.N, s.H, s.W), "A"), ctypes.byref(s.c()),
                              _dev(K, torch.float32, (s.N, OH, OW), "K"), _stream()), "xnor_box_filter_K")
    return K


def xnor_conv2d_chain_workspace_bytes(s: Shape) -> int:
    n = ctypes.c_size_t()
    _ok(lib.xnor_conv2d_chain_workspace_bytes(ctypes.byref(s.c()), ctypes.byref(n)), "xnor_conv2d_chain_workspace_bytes")
    return n.value


def xnor_conv2d_fwd_chain(Ipk: torch.Tensor, Wpk: torch.Tensor | None, K: torch.Tensor | None, alpha: torch.Tensor,
                          s: Shape, Opk: torch.Tensor | None = None, A_next: torch.Tensor | None = None,
                          workspace: torch.Tensor | None = None, A: torch.Tensor | None = None):
    """Returns (Opk int32-typed words [N][OH][OW][ceil(F/32)], A_next fp32 [N][OH][OW]).  Exactly one of
    K and A (this layer's channel mean) is given; Wpk None: the filters are already expanded at the
    start of `workspace` (xnor_filter_expand / xnor_prepare on a buffer of xnor_conv2d_chain_workspace_bytes)."""
    OH, OW = xnor_out_dim(s)
    Cwn = (s.F + 31) // 32
    if Opk is None:
        Opk = torch.empty((s.N, OH, OW, Cwn), dtype=torch.int32, device=Ipk.device)
    if A_next is None:
        A_next = torch.empty((s.N, OH, OW), dtype=torch.float32, device=Ipk.device)
    if workspace is None:
        if Wpk is None:
            raise ValueError("xnor_conv2d_fwd_chain: without Wpk the workspace with the expanded filters is needed")
        workspace = torch.empty((xnor_conv2d_chain_workspace_bytes(s),), dtype=torch.uint8, device=Ipk.device)
    _ok(lib.xnor_conv2d_fwd_chain(
        _dev(Ipk, torch.int32, (s.N, s.H, s.W, s.Cw), "Ipk"),
        _dev(Wpk, torch.int32, (s.F, s.kh, s.kw, s.Cw), "Wpk") if Wpk is not None else None,
        _dev(K, torch.float32, (s.N, OH, OW), "K") if K is not None else None,
        _dev(A, torch.float32, (s.N, s.H, s.W), "A") if A is not None else None,
        _dev(alpha, torch.float32, (s.F,), "alpha"), ctypes.byref(s.c()),
        _dev(Opk, torch.int32, (s.N, OH, OW, Cwn), "Opk"), _dev(A_next, torch.float32, (s.N, OH, OW), "A_next"),
        _dev(workspace, torch.uint8, name="workspace"), workspace.numel(), _stream()), "xnor_conv2d_fwd_chain")
    return Opk, A_next
