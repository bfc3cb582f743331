"""Thin Python binding of include/hdqt.h: argument marshalling only.

Every step of the path runs inside libhdqt.so (hand-written HIP for gfx950).
PyTorch is used for device memory and streams; nothing here computes.  If the
library is missing the import of a function fails loudly: there is no CPU or
PyTorch fallback.
"""
import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Optional

import torch

ROUND_NEAREST, ROUND_STOCHASTIC = 0, 1
GEMM_FWD, GEMM_BWD_INPUT, GEMM_BWD_WEIGHT = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhdqt.so")

EXPORTED = [
    "hdqt_n_eff", "hdqt_codes_pitch", "hdqt_quantize_workspace_size", "hdqt_workspace_layout",
    "hdqt_workspace_size", "hdqt_quantize", "hdqt_gemm_codes", "hdqt_gemm_fwd",
    "hdqt_gemm_bwd_input", "hdqt_gemm_bwd_weight", "hdqt_strerror", "hdqt_last_hip_error",
    "hdqt_profile_enable", "hdqt_profile_collect", "hdqt_quantize_dual",
    "hdqt_quantize_dual_workspace_size", "hdqt_layer_step_workspace_size", "hdqt_layer_step",
    "hdqt_gemm_codes_workspace_size", "hdqt_layer_saved_size", "hdqt_layer_fwd_workspace_size",
    "hdqt_layer_fwd", "hdqt_layer_bwd_workspace_size", "hdqt_layer_bwd",
    "hdqt_gemm_codes_requant_workspace_size", "hdqt_gemm_codes_requant_workspace_size_for",
    "hdqt_gemm_codes_requant",
    "hdqt_gemm_requant_workspace_size", "hdqt_gemm_requant", "hdqt_gemm_codes_bf16",
    "hdqt_gemm_bwd_input_bf16", "hdqt_quantize_dual_im2col", "hdqt_conv_step_workspace_size",
    "hdqt_conv_step", "hdqt_conv_fwd", "hdqt_conv_bwd", "hdqt_gemm_codes_fold", "hdqt_im2col",
    "hdqt_gemm_fwd_static", "hdqt_gemm_fwd_static_max_bytes",
    "hdqt_gemm_bwd_input_masked", "hdqt_layer_bwd_masked", "hdqt_conv_bwd_masked",
    "hdqt_probe_matrix_clock", "hdqt_wall_clock_khz",
]


class HdqtError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


class COperand(C.Structure):
    _fields_ = [("b", C.c_int32), ("round", C.c_int32), ("clip", C.c_float),
                ("tensor_id", C.c_uint32)]


class CParams(C.Structure):
    _fields_ = [("had_block", C.c_int32), ("acc_bits", C.c_int32), ("s", C.c_int64),
                ("seed", C.c_uint64), ("A", COperand), ("B", COperand)]


class CConv(C.Structure):
    _fields_ = [("batch", C.c_int64), ("channels", C.c_int32), ("height", C.c_int32),
                ("width", C.c_int32), ("kh", C.c_int32), ("kw", C.c_int32)]


class CLayout(C.Structure):
    _fields_ = [("scaleA", C.c_size_t), ("scaleB", C.c_size_t), ("codesA", C.c_size_t),
                ("codesB", C.c_size_t), ("acc", C.c_size_t), ("total", C.c_size_t),
                ("RA", C.c_int64), ("RB", C.c_int64), ("D", C.c_int64), ("n_eff", C.c_int32)]


class CKernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64), ("total_ms", C.c_double)]


@dataclass
class Operand:
    b: int = 4
    round: int = ROUND_NEAREST
    clip: float = 1.0
    tensor_id: int = 0

    def c(self) -> COperand:
        return COperand(self.b, self.round, self.clip, self.tensor_id)


@dataclass
class Params:
    had_block: int = 64
    acc_bits: int = 8
    s: int = 32
    seed: int = 0
    A: Operand = field(default_factory=Operand)
    B: Operand = field(default_factory=Operand)

    def c(self) -> CParams:
        return CParams(self.had_block, self.acc_bits, self.s, self.seed, self.A.c(), self.B.c())


_lib = None


def load() -> C.CDLL:
    """Load libhdqt.so (built by paper_2310_03675_amd.build).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2310_03675_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
    lib.hdqt_n_eff.restype = i32
    lib.hdqt_n_eff.argtypes = [i64, i32]
    lib.hdqt_codes_pitch.restype = i64
    lib.hdqt_codes_pitch.argtypes = [i64, i32]
    lib.hdqt_quantize_workspace_size.restype = sz
    lib.hdqt_quantize_workspace_size.argtypes = []
    lib.hdqt_workspace_layout.restype = i32
    lib.hdqt_workspace_layout.argtypes = [i32, i64, i64, i64, C.POINTER(CParams), C.POINTER(CLayout)]
    lib.hdqt_workspace_size.restype = sz
    lib.hdqt_workspace_size.argtypes = [i32, i64, i64, i64, C.POINTER(CParams)]
    lib.hdqt_quantize.restype = i32
    lib.hdqt_quantize.argtypes = [vp, i64, i64, i32, i32, C.POINTER(COperand), C.c_uint64, vp, vp,
                                  vp, sz, vp]
    lib.hdqt_quantize_dual_workspace_size.restype = sz
    lib.hdqt_quantize_dual_workspace_size.argtypes = []
    lib.hdqt_gemm_codes_workspace_size.restype = sz
    lib.hdqt_gemm_codes_workspace_size.argtypes = [i64, i64, i64, i64]
    lib.hdqt_gemm_codes_requant_workspace_size.restype = sz
    lib.hdqt_gemm_codes_requant_workspace_size.argtypes = [i64, i64, i64, i64]
    lib.hdqt_gemm_codes_requant_workspace_size_for.restype = sz
    lib.hdqt_gemm_codes_requant_workspace_size_for.argtypes = [i64, i64, i64, i64, i32, i32, i32]
    lib.hdqt_gemm_codes_requant.restype = i32
    lib.hdqt_gemm_codes_requant.argtypes = [vp, vp, i32, i32, vp, vp, i64, i64, i64, i32, i32, i64, vp, vp,
                                            vp, sz, vp]
    lib.hdqt_gemm_requant_workspace_size.restype = sz
    lib.hdqt_gemm_requant_workspace_size.argtypes = [i32, i64, i64, i64, C.POINTER(CParams)]
    lib.hdqt_gemm_requant.restype = i32
    lib.hdqt_gemm_requant.argtypes = [i32, vp, vp, vp, i64, i64, i64, C.POINTER(CParams), vp, vp, sz, vp]
    lib.hdqt_layer_saved_size.restype = sz
    lib.hdqt_layer_saved_size.argtypes = [i64, i64, C.POINTER(CParams)]
    lib.hdqt_layer_fwd_workspace_size.restype = sz
    lib.hdqt_layer_fwd_workspace_size.argtypes = [i64, i64, i64] + [C.POINTER(CParams)] * 2
    lib.hdqt_layer_fwd.restype = i32
    lib.hdqt_layer_fwd.argtypes = [vp] * 3 + [i64, i64, i64] + [C.POINTER(CParams)] * 2 + [vp, sz, vp, sz, vp]
    lib.hdqt_layer_bwd_workspace_size.restype = sz
    lib.hdqt_layer_bwd_workspace_size.argtypes = [i64, i64, i64] + [C.POINTER(CParams)] * 2
    lib.hdqt_layer_bwd.restype = i32
    lib.hdqt_layer_bwd.argtypes = [vp] * 5 + [i64, i64, i64] + [C.POINTER(CParams)] * 2 + [vp, sz, vp]
    lib.hdqt_layer_step_workspace_size.restype = sz
    lib.hdqt_layer_step_workspace_size.argtypes = [i64, i64, i64] + [C.POINTER(CParams)] * 3
    lib.hdqt_layer_step.restype = i32
    lib.hdqt_layer_step.argtypes = [vp] * 6 + [i64, i64, i64] + [C.POINTER(CParams)] * 3 + [vp, sz, vp]
    lib.hdqt_quantize_dual.restype = i32
    lib.hdqt_quantize_dual.argtypes = [vp, i64, i64, i32, C.POINTER(COperand), C.POINTER(COperand),
                                       C.c_uint64, vp, vp, vp, vp, vp, sz, vp]
    lib.hdqt_gemm_codes.restype = i32
    lib.hdqt_gemm_codes.argtypes = [vp, vp, i32, i32, vp, vp, i64, i64, i64, i32, i32, i64, vp, vp,
                                    vp, sz, vp]
    lib.hdqt_quantize_dual_im2col.restype = i32
    lib.hdqt_quantize_dual_im2col.argtypes = [vp, C.POINTER(CConv), i32, C.POINTER(COperand),
                                              C.POINTER(COperand), C.c_uint64, vp, vp, vp, vp, vp, sz, vp]
    lib.hdqt_conv_step_workspace_size.restype = sz
    lib.hdqt_conv_step_workspace_size.argtypes = [C.POINTER(CConv), i64] + [C.POINTER(CParams)] * 3
    lib.hdqt_conv_step.restype = i32
    lib.hdqt_conv_step.argtypes = [vp, C.POINTER(CConv), vp, vp, vp, vp, vp, i64] + [C.POINTER(CParams)] * 3 + [vp, sz, vp]
    lib.hdqt_conv_fwd.restype = i32
    lib.hdqt_conv_fwd.argtypes = [vp, C.POINTER(CConv), vp, vp, i64] + [C.POINTER(CParams)] * 2 + [vp, sz, vp, sz, vp]
    lib.hdqt_conv_bwd.restype = i32
    lib.hdqt_conv_bwd.argtypes = [vp, vp, vp, C.POINTER(CConv), vp, vp, i64] + [C.POINTER(CParams)] * 2 + [vp, sz, vp]
    lib.hdqt_gemm_codes_fold.restype = i32
    lib.hdqt_gemm_codes_fold.argtypes = [vp, vp, i32, i32, vp, vp, C.POINTER(CConv), i64, i32, i32, i64, vp, vp]
    lib.hdqt_im2col.restype = i32
    lib.hdqt_im2col.argtypes = [vp, i64] + [i32] * 8 + [vp, vp]
    lib.hdqt_gemm_codes_bf16.restype = i32
    lib.hdqt_gemm_codes_bf16.argtypes = lib.hdqt_gemm_codes.argtypes
    for name in ("hdqt_gemm_fwd", "hdqt_gemm_bwd_input", "hdqt_gemm_bwd_weight", "hdqt_gemm_bwd_input_bf16"):
        fn = getattr(lib, name)
        fn.restype = i32
        fn.argtypes = [vp, vp, vp, i64, i64, i64, C.POINTER(CParams), vp, vp, sz, vp]
    lib.hdqt_gemm_bwd_input_masked.restype = i32
    lib.hdqt_gemm_bwd_input_masked.argtypes = [vp, vp, vp, vp, i64, i64, i64, C.POINTER(CParams), vp, vp, sz, vp]
    lib.hdqt_layer_bwd_masked.restype = i32
    lib.hdqt_layer_bwd_masked.argtypes = [vp] * 6 + [i64, i64, i64] + [C.POINTER(CParams)] * 2 + [vp, sz, vp]
    lib.hdqt_conv_bwd_masked.restype = i32
    lib.hdqt_conv_bwd_masked.argtypes = [vp, vp, vp, C.POINTER(CConv), vp, vp, vp, i64] + [C.POINTER(CParams)] * 2 + [vp, sz, vp]
    lib.hdqt_wall_clock_khz.restype = i32
    lib.hdqt_wall_clock_khz.argtypes = []
    lib.hdqt_probe_matrix_clock.restype = i32
    lib.hdqt_probe_matrix_clock.argtypes = [vp, i32, i32, vp, vp, sz, vp]
    lib.hdqt_gemm_fwd_static.restype = i32
    lib.hdqt_gemm_fwd_static.argtypes = [vp, vp, vp, i64, i64, i64, C.POINTER(CParams), vp, vp]
    lib.hdqt_gemm_fwd_static_max_bytes.restype = sz
    lib.hdqt_gemm_fwd_static_max_bytes.argtypes = []
    lib.hdqt_strerror.restype = C.c_char_p
    lib.hdqt_strerror.argtypes = [i32]
    lib.hdqt_last_hip_error.restype = i32
    lib.hdqt_last_hip_error.argtypes = []
    lib.hdqt_profile_enable.restype = i32
    lib.hdqt_profile_enable.argtypes = [i32]
    lib.hdqt_profile_collect.restype = i32
    lib.hdqt_profile_collect.argtypes = [C.POINTER(CKernelTime), i32]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().hdqt_strerror(code).decode()


def profile_enable(on: bool) -> None:
    load().hdqt_profile_enable(1 if on else 0)


def profile_collect() -> dict:
    """-> {kernel name: (launches, total milliseconds)} since the last collect."""
    rows = (CKernelTime * 32)()
    n = load().hdqt_profile_collect(rows, 32)
    return {rows[i].name.decode(): (rows[i].launches, rows[i].total_ms) for i in range(min(n, 32))}


def n_eff(D: int, had_block: int) -> int:
    return load().hdqt_n_eff(D, had_block)


def codes_pitch(D: int, b: int) -> int:
    return load().hdqt_codes_pitch(D, b)


def workspace_layout(kind: int, M: int, K: int, N: int, params: Params) -> CLayout:
    L = CLayout()
    p = params.c()
    rc = load().hdqt_workspace_layout(kind, M, K, N, C.byref(p), C.byref(L))
    if rc:
        raise HdqtError(rc, "hdqt_workspace_layout")
    return L


def workspace_size(kind: int, M: int, K: int, N: int, params: Params) -> int:
    p = params.c()
    return load().hdqt_workspace_size(kind, M, K, N, C.byref(p))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream: Optional[torch.cuda.Stream]):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _check_dev(*tensors):
    for t in tensors:
        if t is not None and not (t.is_cuda and t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def quantize(T: torch.Tensor, axis: int, had_block: int, op: Operand, seed: int = 0,
             stream: Optional[torch.cuda.Stream] = None):
    """hdqt_quantize -> (codes uint8 [lines, pitch], scale float32 [1]) on the device."""
    _check_dev(T)
    assert T.dtype == torch.float32 and T.dim() == 2
    rows, cols = T.shape
    D, lines = (cols, rows) if axis == 1 else (rows, cols)
    pitch = codes_pitch(D, op.b)
    codes = torch.empty((lines, pitch), dtype=torch.uint8, device=T.device)
    scale = torch.empty(1, dtype=torch.float32, device=T.device)
    ws = torch.empty(load().hdqt_quantize_workspace_size(), dtype=torch.uint8, device=T.device)
    cop = op.c()
    rc = load().hdqt_quantize(_ptr(T), rows, cols, axis, had_block, C.byref(cop), seed,
                              _ptr(codes), _ptr(scale), _ptr(ws), ws.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_quantize")
    return codes, scale


def quantize_dual(T: torch.Tensor, had_block: int, op_axis1: Operand, op_axis0: Operand, seed: int = 0,
                  out=None, workspace: Optional[torch.Tensor] = None,
                  stream: Optional[torch.cuda.Stream] = None):
    """hdqt_quantize_dual -> (codes_axis1, scale_axis1, codes_axis0, scale_axis0).
    `out` may carry preallocated (codes1, scale1, codes0, scale0)."""
    _check_dev(T)
    assert T.dtype == torch.float32 and T.dim() == 2
    rows, cols = T.shape
    if out is None:
        out = (torch.empty((rows, codes_pitch(cols, op_axis1.b)), dtype=torch.uint8, device=T.device),
               torch.empty(1, dtype=torch.float32, device=T.device),
               torch.empty((cols, codes_pitch(rows, op_axis0.b)), dtype=torch.uint8, device=T.device),
               torch.empty(1, dtype=torch.float32, device=T.device))
    c1, s1, c0, s0 = out
    if workspace is None:
        workspace = torch.empty(load().hdqt_quantize_dual_workspace_size(), dtype=torch.uint8,
                                device=T.device)
    o1, o0 = op_axis1.c(), op_axis0.c()
    rc = load().hdqt_quantize_dual(_ptr(T), rows, cols, had_block, C.byref(o1), C.byref(o0), seed,
                                   _ptr(c1), _ptr(s1), _ptr(c0), _ptr(s0), _ptr(workspace),
                                   workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_quantize_dual")
    return c1, s1, c0, s0


def im2col(act: torch.Tensor, kh: int, kw: int, stride: int = 1, pad_h: int = 0, pad_w: int = 0,
           stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """hdqt_im2col -> X [batch*Ho*Wo, C*kh*kw] (column index c*kh*kw + ty*kw + tx)."""
    assert act.dim() == 4 and act.dtype == torch.float32
    act = act.contiguous()
    _check_dev(act)
    b, c, h, w = act.shape
    Ho, Wo = (h + 2 * pad_h - kh) // stride + 1, (w + 2 * pad_w - kw) // stride + 1
    X = torch.empty((b * Ho * Wo, c * kh * kw), dtype=torch.float32, device=act.device)
    rc = load().hdqt_im2col(_ptr(act), b, c, h, w, kh, kw, stride, pad_h, pad_w, _ptr(X), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_im2col")
    return X


def conv_geometry(act: torch.Tensor, kh: int, kw: int) -> CConv:
    """Geometry of a stride-1, same-size convolution over act [batch, C, H, W]."""
    assert act.dim() == 4 and act.dtype == torch.float32 and act.is_contiguous()
    b, c, h, w = act.shape
    return CConv(b, c, h, w, kh, kw)


def quantize_dual_im2col(act: torch.Tensor, kh: int, kw: int, had_block: int, op_axis1: Operand,
                         op_axis0: Operand, seed: int = 0, stream: Optional[torch.cuda.Stream] = None):
    """hdqt_quantize_dual_im2col -> (codes_axis1, scale_axis1, codes_axis0, scale_axis0) of the
    im2col matrix [batch*H*W, C*kh*kw] of act, which is never formed."""
    _check_dev(act)
    geo = conv_geometry(act, kh, kw)
    rows, cols = act.shape[0] * act.shape[2] * act.shape[3], act.shape[1] * kh * kw
    c1 = torch.empty((rows, codes_pitch(cols, op_axis1.b)), dtype=torch.uint8, device=act.device)
    c0 = torch.empty((cols, codes_pitch(rows, op_axis0.b)), dtype=torch.uint8, device=act.device)
    s1 = torch.empty(1, dtype=torch.float32, device=act.device)
    s0 = torch.empty(1, dtype=torch.float32, device=act.device)
    ws = torch.empty(load().hdqt_quantize_dual_workspace_size(), dtype=torch.uint8, device=act.device)
    o1, o0 = op_axis1.c(), op_axis0.c()
    rc = load().hdqt_quantize_dual_im2col(_ptr(act), C.byref(geo), had_block, C.byref(o1), C.byref(o0),
                                          seed, _ptr(c1), _ptr(s1), _ptr(c0), _ptr(s0), _ptr(ws),
                                          ws.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_quantize_dual_im2col")
    return c1, s1, c0, s0


def conv_step(act: torch.Tensor, kh: int, kw: int, W: torch.Tensor, G: torch.Tensor, fwd: Params,
              bwd_input: Params, bwd_weight: Params, out=None, workspace: Optional[torch.Tensor] = None,
              stream: Optional[torch.cuda.Stream] = None):
    """hdqt_conv_step -> (Z [M, N], dXcol [M, K], dW [K, N], workspace)."""
    _check_dev(act, W, G, workspace)
    geo = conv_geometry(act, kh, kw)
    M, K, N = act.shape[0] * act.shape[2] * act.shape[3], act.shape[1] * kh * kw, W.shape[1]
    pf, pi, pw = fwd.c(), bwd_input.c(), bwd_weight.c()
    if workspace is None:
        need = load().hdqt_conv_step_workspace_size(C.byref(geo), N, C.byref(pf), C.byref(pi), C.byref(pw))
        if need == 0:
            raise HdqtError(-13, "hdqt_conv_step_workspace_size")
        workspace = torch.empty(need, dtype=torch.uint8, device=act.device)
    if out is None:
        out = (torch.empty((M, N), dtype=torch.float32, device=act.device),
               torch.empty((M, K), dtype=torch.float32, device=act.device),
               torch.empty((K, N), dtype=torch.float32, device=act.device))
    Z, dX, dW = out
    rc = load().hdqt_conv_step(_ptr(act), C.byref(geo), _ptr(W), _ptr(G), _ptr(Z), _ptr(dX), _ptr(dW), N,
                               C.byref(pf), C.byref(pi), C.byref(pw), _ptr(workspace), workspace.numel(),
                               _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_conv_step")
    return Z, dX, dW, workspace


def gemm_codes(qA: torch.Tensor, qB: torch.Tensor, bA: int, bB: int, scaleA: torch.Tensor,
               scaleB: torch.Tensor, D: int, n: int, acc_bits: int, s: int,
               want_out: bool = True, want_acc: bool = True,
               workspace: Optional[torch.Tensor] = None,
               out: Optional[torch.Tensor] = None, acc: Optional[torch.Tensor] = None,
               stream: Optional[torch.cuda.Stream] = None, bf16: bool = False):
    """hdqt_gemm_codes -> (out fp32 [RA, RB] | None, acc int32 [RA, RB] | None);
    with bf16=True hdqt_gemm_codes_bf16 and `out` is a torch.bfloat16 tensor."""
    _check_dev(qA, qB, scaleA, scaleB)
    RA, RB = qA.shape[0], qB.shape[0]
    fn = "hdqt_gemm_codes_bf16" if bf16 else "hdqt_gemm_codes"
    if out is None and want_out:
        out = torch.empty((RA, RB), dtype=torch.bfloat16 if bf16 else torch.float32, device=qA.device)
    assert out is None or out.dtype == (torch.bfloat16 if bf16 else torch.float32)
    if acc is None and want_acc:
        acc = torch.empty((RA, RB), dtype=torch.int32, device=qA.device)
    if workspace is None:
        need = load().hdqt_gemm_codes_workspace_size(RA, RB, D, s)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=qA.device)
    rc = getattr(load(), fn)(_ptr(qA), _ptr(qB), bA, bB, _ptr(scaleA), _ptr(scaleB), RA, RB, D,
                             n, acc_bits, s, _ptr(out), _ptr(acc), _ptr(workspace),
                             workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, fn)
    return out, acc


_GEMM_FN = {GEMM_FWD: "hdqt_gemm_fwd", GEMM_BWD_INPUT: "hdqt_gemm_bwd_input",
            GEMM_BWD_WEIGHT: "hdqt_gemm_bwd_weight"}


def out_shape(kind: int, M: int, K: int, N: int):
    return {GEMM_FWD: (M, N), GEMM_BWD_INPUT: (M, K), GEMM_BWD_WEIGHT: (K, N)}[kind]


def gemm(kind: int, P: torch.Tensor, Q: torch.Tensor, M: int, K: int, N: int, params: Params,
         out: Optional[torch.Tensor] = None, acc: Optional[torch.Tensor] = None,
         want_acc: bool = False, workspace: Optional[torch.Tensor] = None,
         stream: Optional[torch.cuda.Stream] = None, bf16: bool = False,
         mask: Optional[torch.Tensor] = None):
    """hdqt_gemm_{fwd,bwd_input,bwd_weight}.  P, Q are the two source tensors of
    `kind`: (X, W), (G, W), (X, G).  -> (out, acc | None, workspace).  bf16=True (input
    gradient only): hdqt_gemm_bwd_input_bf16, `out` is a torch.bfloat16 tensor.  mask (input
    gradient only): hdqt_gemm_bwd_input_masked, the layer's input X [M, K]."""
    _check_dev(P, Q, out, acc, workspace, mask)
    shape = out_shape(kind, M, K, N)
    assert not bf16 or kind == GEMM_BWD_INPUT
    fn = "hdqt_gemm_bwd_input_bf16" if bf16 else _GEMM_FN[kind]
    if out is None:
        out = torch.empty(shape, dtype=torch.bfloat16 if bf16 else torch.float32, device=P.device)
    assert out.dtype == (torch.bfloat16 if bf16 else torch.float32)
    if acc is None and want_acc:
        acc = torch.empty(shape, dtype=torch.int32, device=P.device)
    p = params.c()
    need = load().hdqt_workspace_size(kind, M, K, N, C.byref(p))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=P.device)
    if mask is not None:
        assert kind == GEMM_BWD_INPUT and not bf16 and tuple(mask.shape) == tuple(shape) and mask.dtype == torch.float32
        fn = "hdqt_gemm_bwd_input_masked"
        rc = load().hdqt_gemm_bwd_input_masked(_ptr(P), _ptr(Q), _ptr(mask), _ptr(out), M, K, N, C.byref(p),
                                               _ptr(acc), _ptr(workspace), workspace.numel(), _stream(stream))
    else:
        rc = getattr(load(), fn)(_ptr(P), _ptr(Q), _ptr(out), M, K, N, C.byref(p),
                                 _ptr(acc), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, fn)
    return out, acc, workspace


def probe_matrix_clock(fragments: torch.Tensor, iters: int = 4000, waves_per_simd: int = 2):
    """hdqt_probe_matrix_clock -> dict: the matrix pipe's rate on the given operand fragments
    (8 KiB uint8 on the device) and the shader clock under that load.  The rate is taken from
    the whole launch's duration (HIP events): waves_per_simd waves x 16 * iters MFMAs on each of
    the chip's 1024 SIMDs; the clock from one wave's cycle and wall-clock counters."""
    _check_dev(fragments)
    assert fragments.dtype == torch.uint8 and fragments.numel() >= 8192
    result = torch.zeros(2, dtype=torch.int64, device=fragments.device)
    scratch = torch.empty(1 << 20, dtype=torch.uint8, device=fragments.device)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for rep in range(2):       # the first launch warms the clock up
        if rep == 1:
            e0.record()
        rc = load().hdqt_probe_matrix_clock(_ptr(fragments), iters, waves_per_simd, _ptr(result), _ptr(scratch),
                                            scratch.numel(), _stream(None))
        if rc:
            raise HdqtError(rc, "hdqt_probe_matrix_clock")
    e1.record()
    torch.cuda.synchronize()
    cycles, ticks = (int(v) for v in result.cpu())
    wall_khz = load().hdqt_wall_clock_khz() or 100000
    mhz = cycles / (ticks * 1e3 / wall_khz)
    ns_per_mfma = e0.elapsed_time(e1) * 1e6 / (waves_per_simd * 16.0 * iters)       # per SIMD
    return {"waves_per_simd": waves_per_simd, "shader_clock_mhz": mhz, "ns_per_mfma_per_simd": ns_per_mfma,
            "cycles_per_mfma_per_simd": ns_per_mfma * mhz * 1e-3,
            "TOPs": 65536.0 * 1024.0 / ns_per_mfma / 1e3,
            "frac_of_published_peak": 65536.0 * 1024.0 / ns_per_mfma / 1e3 / 5000.0}


def gemm_fwd_static(X: torch.Tensor, W: torch.Tensor, params: Params, out: torch.Tensor,
                    acc: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """hdqt_gemm_fwd_static: the forward matmul without a workspace; the caller brings the
    output (nothing is allocated here either)."""
    _check_dev(X, W, out, acc)
    M, K = X.shape
    N = W.shape[1]
    assert tuple(out.shape) == (M, N) and out.dtype == torch.float32
    p = params.c()
    rc = load().hdqt_gemm_fwd_static(_ptr(X), _ptr(W), _ptr(out), M, K, N, C.byref(p), _ptr(acc),
                                     _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_gemm_fwd_static")
    return out


def gemm_fwd(X, W, params: Params, **kw):
    M, K = X.shape
    return gemm(GEMM_FWD, X, W, M, K, W.shape[1], params, **kw)


def gemm_bwd_input(G, W, params: Params, **kw):
    M, N = G.shape
    return gemm(GEMM_BWD_INPUT, G, W, M, W.shape[0], N, params, **kw)


def gemm_bwd_weight(X, G, params: Params, **kw):
    M, K = X.shape
    return gemm(GEMM_BWD_WEIGHT, X, G, M, K, G.shape[1], params, **kw)


def layer_step_workspace_size(M: int, K: int, N: int, fwd: Params, bwd_input: Optional[Params],
                              bwd_weight: Params) -> int:
    pf, pw = fwd.c(), bwd_weight.c()
    pi = bwd_input.c() if bwd_input is not None else None
    return load().hdqt_layer_step_workspace_size(M, K, N, C.byref(pf),
                                                 C.byref(pi) if pi is not None else None, C.byref(pw))


def layer_step(X: torch.Tensor, W: torch.Tensor, G: torch.Tensor, fwd: Params,
               bwd_input: Optional[Params], bwd_weight: Params, out=None,
               workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """hdqt_layer_step -> (Z, dX | None, dW, workspace).  dX is skipped when
    `bwd_input` is None.  `out` may carry preallocated (Z, dX, dW)."""
    _check_dev(X, W, G, workspace)
    M, K = X.shape
    N = W.shape[1]
    assert W.shape[0] == K and tuple(G.shape) == (M, N)
    if out is None:
        new = lambda *shape: torch.empty(shape, dtype=torch.float32, device=X.device)
        out = (new(M, N), new(M, K) if bwd_input is not None else None, new(K, N))
    Z, dX, dW = out
    if workspace is None:
        need = layer_step_workspace_size(M, K, N, fwd, bwd_input, bwd_weight)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    pf, pw = fwd.c(), bwd_weight.c()
    pi = bwd_input.c() if bwd_input is not None else None
    rc = load().hdqt_layer_step(_ptr(X), _ptr(W), _ptr(G), _ptr(Z), _ptr(dX), _ptr(dW), M, K, N,
                                C.byref(pf), C.byref(pi) if pi is not None else None, C.byref(pw),
                                _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_layer_step")
    return Z, dX, dW, workspace


def _byref(p):
    return C.byref(p) if p is not None else None


def layer_fwd(X: torch.Tensor, W: torch.Tensor, fwd: Params, bwd_weight: Optional[Params] = None,
              out: Optional[torch.Tensor] = None, saved: Optional[torch.Tensor] = None,
              workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """hdqt_layer_fwd -> (Z, saved | None).  With `bwd_weight`, `saved` receives X's codes
    along M for layer_bwd (a uint8 tensor of hdqt_layer_saved_size bytes)."""
    _check_dev(X, W, out, saved, workspace)
    M, K = X.shape
    N = W.shape[1]
    assert W.shape[0] == K
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=X.device)
    pf = fwd.c()
    pw = bwd_weight.c() if bwd_weight is not None else None
    if pw is not None and saved is None:
        saved = torch.empty(load().hdqt_layer_saved_size(M, K, C.byref(pw)), dtype=torch.uint8,
                            device=X.device)
    if workspace is None:
        need = load().hdqt_layer_fwd_workspace_size(M, K, N, C.byref(pf), _byref(pw))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    rc = load().hdqt_layer_fwd(_ptr(X), _ptr(W), _ptr(out), M, K, N, C.byref(pf), _byref(pw),
                               _ptr(saved), saved.numel() if saved is not None else 0,
                               _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_layer_fwd")
    return out, saved


def conv_fwd(act: torch.Tensor, kh: int, kw: int, W: torch.Tensor, fwd: Params, bwd_weight: Params,
             stream: Optional[torch.cuda.Stream] = None):
    """hdqt_conv_fwd -> (Z [batch*H*W, N], saved): hdqt_layer_fwd with X given as the activation.
    Raises HdqtError with code -13 for geometries the activation-source kernels do not take."""
    _check_dev(act, W)
    geo = conv_geometry(act, kh, kw)
    M, K, N = act.shape[0] * act.shape[2] * act.shape[3], act.shape[1] * kh * kw, W.shape[1]
    assert W.shape[0] == K
    pf, pw = fwd.c(), bwd_weight.c()
    out = torch.empty((M, N), dtype=torch.float32, device=act.device)
    saved = torch.empty(load().hdqt_layer_saved_size(M, K, C.byref(pw)), dtype=torch.uint8, device=act.device)
    need = load().hdqt_layer_fwd_workspace_size(M, K, N, C.byref(pf), C.byref(pw))
    workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=act.device)
    rc = load().hdqt_conv_fwd(_ptr(act), C.byref(geo), _ptr(W), _ptr(out), N, C.byref(pf), C.byref(pw),
                              _ptr(saved), saved.numel(), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_conv_fwd")
    return out, saved


def conv_bwd(G: torch.Tensor, W: torch.Tensor, saved: torch.Tensor, act_shape, kh: int, kw: int,
             bwd_input: Params, bwd_weight: Params, stream: Optional[torch.cuda.Stream] = None,
             mask: Optional[torch.Tensor] = None):
    """hdqt_conv_bwd -> (dAct [batch, C, H, W], dW [K, N]): hdqt_layer_bwd with the input gradient
    folded back onto the activation inside the matmul.  HdqtError -13 for geometries not taken.
    mask: hdqt_conv_bwd_masked, the activation itself (dAct is written where it is positive)."""
    _check_dev(G, W, saved, mask)
    batch, Cin, H, Wd = act_shape
    geo = CConv(batch, Cin, H, Wd, kh, kw)
    M, K, N = batch * H * Wd, Cin * kh * kw, G.shape[1]
    assert tuple(G.shape) == (M, N) and tuple(W.shape) == (K, N)
    pi, pw = bwd_input.c(), bwd_weight.c()
    dAct = torch.empty((batch, Cin, H, Wd), dtype=torch.float32, device=G.device)
    dW = torch.empty((K, N), dtype=torch.float32, device=G.device)
    need = load().hdqt_layer_bwd_workspace_size(M, K, N, C.byref(pi), C.byref(pw))
    workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=G.device)
    if mask is not None:
        assert tuple(mask.shape) == tuple(dAct.shape) and mask.dtype == torch.float32 and mask.is_contiguous()
        rc = load().hdqt_conv_bwd_masked(_ptr(G), _ptr(W), _ptr(saved), C.byref(geo), _ptr(mask), _ptr(dAct),
                                         _ptr(dW), N, C.byref(pi), C.byref(pw), _ptr(workspace),
                                         workspace.numel(), _stream(stream))
    else:
        rc = load().hdqt_conv_bwd(_ptr(G), _ptr(W), _ptr(saved), C.byref(geo), _ptr(dAct), _ptr(dW), N,
                                  C.byref(pi), C.byref(pw), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_conv_bwd")
    return dAct, dW


def gemm_codes_fold(qG: torch.Tensor, qW: torch.Tensor, bG: int, bW: int, scaleG: torch.Tensor,
                    scaleW: torch.Tensor, act_shape, kh: int, kw: int, n: int, acc_bits: int, s: int,
                    out: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """hdqt_gemm_codes_fold -> dAct [batch, C, H, W]."""
    _check_dev(qG, qW, scaleG, scaleW)
    batch, Cin, H, Wd = act_shape
    geo = CConv(batch, Cin, H, Wd, kh, kw)
    N = qG.shape[1] * (2 if bG <= 4 else 1)
    if out is None:
        out = torch.empty((batch, Cin, H, Wd), dtype=torch.float32, device=qG.device)
    rc = load().hdqt_gemm_codes_fold(_ptr(qG), _ptr(qW), bG, bW, _ptr(scaleG), _ptr(scaleW), C.byref(geo), N,
                                     n, acc_bits, s, _ptr(out), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_gemm_codes_fold")
    return out


def layer_bwd(G: torch.Tensor, W: torch.Tensor, saved: torch.Tensor, K: int,
              bwd_input: Optional[Params], bwd_weight: Params, out=None,
              workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
              mask: Optional[torch.Tensor] = None):
    """hdqt_layer_bwd -> (dX | None, dW).  dX is skipped when `bwd_input` is None.
    `out` may carry preallocated (dX, dW).  mask: hdqt_layer_bwd_masked, the layer's input
    X [M, K] (dX is written where it is positive, zero elsewhere)."""
    _check_dev(G, W, saved, workspace, mask)
    M, N = G.shape
    if out is None:
        new = lambda *shape: torch.empty(shape, dtype=torch.float32, device=G.device)
        out = (new(M, K) if bwd_input is not None else None, new(K, N))
    dX, dW = out
    pi = bwd_input.c() if bwd_input is not None else None
    pw = bwd_weight.c()
    if workspace is None:
        need = load().hdqt_layer_bwd_workspace_size(M, K, N, _byref(pi), C.byref(pw))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=G.device)
    if mask is not None:
        assert dX is not None and tuple(mask.shape) == (M, K) and mask.dtype == torch.float32 and mask.is_contiguous()
        rc = load().hdqt_layer_bwd_masked(_ptr(G), _ptr(W), _ptr(saved), _ptr(mask), _ptr(dX), _ptr(dW), M, K, N,
                                          _byref(pi), C.byref(pw), _ptr(workspace), workspace.numel(),
                                          _stream(stream))
    else:
        rc = load().hdqt_layer_bwd(_ptr(G), _ptr(W), _ptr(saved), _ptr(dX), _ptr(dW), M, K, N, _byref(pi),
                                   C.byref(pw), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_layer_bwd")
    return dX, dW


def gemm_codes_requant(qA: torch.Tensor, qB: torch.Tensor, bA: int, bB: int, scaleA: torch.Tensor,
                       scaleB: torch.Tensor, D: int, n: int, acc_bits: int, s: int,
                       want_acc: bool = True, workspace: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None):
    """hdqt_gemm_codes_requant -> (out fp32 [RA, RB], acc int32 [RA, RB] | None)."""
    _check_dev(qA, qB, scaleA, scaleB, workspace)
    RA, RB = qA.shape[0], qB.shape[0]
    out = torch.empty((RA, RB), dtype=torch.float32, device=qA.device)
    acc = torch.empty((RA, RB), dtype=torch.int32, device=qA.device) if want_acc else None
    if workspace is None:
        need = load().hdqt_gemm_codes_requant_workspace_size_for(RA, RB, D, s, bA, bB, acc_bits)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=qA.device)
    rc = load().hdqt_gemm_codes_requant(_ptr(qA), _ptr(qB), bA, bB, _ptr(scaleA), _ptr(scaleB), RA, RB, D,
                                        n, acc_bits, s, _ptr(out), _ptr(acc), _ptr(workspace),
                                        workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_gemm_codes_requant")
    return out, acc


def gemm_requant(kind: int, P: torch.Tensor, Q: torch.Tensor, M: int, K: int, N: int, params: Params,
                 want_acc: bool = False, workspace: Optional[torch.Tensor] = None,
                 stream: Optional[torch.cuda.Stream] = None):
    """hdqt_gemm_requant -> (out, acc | None, workspace); the workspace starts with the
    layout hdqt_workspace_layout describes (scales and codes of both operands)."""
    _check_dev(P, Q, workspace)
    shape = out_shape(kind, M, K, N)
    out = torch.empty(shape, dtype=torch.float32, device=P.device)
    acc = torch.empty(shape, dtype=torch.int32, device=P.device) if want_acc else None
    p = params.c()
    if workspace is None:
        need = load().hdqt_gemm_requant_workspace_size(kind, M, K, N, C.byref(p))
        if need == 0:
            raise HdqtError(-5, "hdqt_gemm_requant_workspace_size")
        workspace = torch.empty(need, dtype=torch.uint8, device=P.device)
    rc = load().hdqt_gemm_requant(kind, _ptr(P), _ptr(Q), _ptr(out), M, K, N, C.byref(p), _ptr(acc),
                                  _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise HdqtError(rc, "hdqt_gemm_requant")
    return out, acc, workspace
