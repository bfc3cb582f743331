"""NumPy front end of the C oracle (oracle/hdqt_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg, never by the product path.  Argument marshalling
only; every number comes out of the C file.
"""
import ctypes as C
import os
from dataclasses import dataclass, field

import numpy as np

from . import build as _build

ROUND_NEAREST = 0
ROUND_STOCHASTIC = 1
FWD, BWD_INPUT, BWD_WEIGHT = 0, 1, 2

_lib = None


class _Operand(C.Structure):
    _fields_ = [("b", C.c_int), ("round_mode", C.c_int), ("clip", C.c_float),
                ("tensor_id", C.c_uint32)]


class _Params(C.Structure):
    _fields_ = [("had_block", C.c_int), ("acc_bits", C.c_int), ("s", C.c_int64),
                ("seed", C.c_uint64), ("A", _Operand), ("B", _Operand)]


@dataclass
class Operand:
    b: int = 4
    round_mode: int = ROUND_NEAREST
    clip: float = 1.0
    tensor_id: int = 0


@dataclass
class Params:
    had_block: int = 64
    acc_bits: int = 8
    s: int = 32
    seed: int = 0
    A: Operand = field(default_factory=Operand)
    B: Operand = field(default_factory=Operand)

    def _c(self):
        return _Params(self.had_block, self.acc_bits, self.s, self.seed,
                       _Operand(self.A.b, self.A.round_mode, self.A.clip, self.A.tensor_id),
                       _Operand(self.B.b, self.B.round_mode, self.B.clip, self.B.tensor_id))


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.orc_n_eff.restype = C.c_int
        _lib.orc_n_eff.argtypes = [C.c_int64, C.c_int]
        _lib.orc_sr_bits.restype = C.c_uint32
        _lib.orc_sr_bits.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64]
        _lib.orc_packed_pitch.restype = C.c_int64
        _lib.orc_packed_pitch.argtypes = [C.c_int64, C.c_int]
        _lib.orc_dequant_factor.restype = C.c_float
        _lib.orc_dequant_factor.argtypes = [C.c_float, C.c_float, C.c_int]
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def n_eff(D: int, n: int) -> int:
    return lib().orc_n_eff(D, n)


def hadamard_matrix(k: int) -> np.ndarray:
    n = 1 << k
    H = np.zeros((n, n), dtype=np.int8)
    lib().orc_hadamard_matrix(C.c_int(k), _p(H, C.c_int8))
    return H


def hadamard_transform(T, axis: int, n: int) -> np.ndarray:
    T = _f32(T)
    rows, cols = T.shape
    Y = np.empty_like(T)
    lib().orc_hadamard_transform(_p(T, C.c_float), C.c_int64(rows), C.c_int64(cols),
                                 C.c_int(axis), C.c_int(n), _p(Y, C.c_float))
    return Y


def hadamard_transform_f64(T, axis: int, n: int) -> np.ndarray:
    T = _f32(T)
    rows, cols = T.shape
    Y = np.empty(T.shape, dtype=np.float64)
    lib().orc_hadamard_transform_f64(_p(T, C.c_float), C.c_int64(rows), C.c_int64(cols),
                                     C.c_int(axis), C.c_int(n), _p(Y, C.c_double))
    return Y


def philox4x32_10(ctr, key) -> np.ndarray:
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(ctr, C.c_uint32), _p(key, C.c_uint32), _p(out, C.c_uint32))
    return out


def sr_bits(seed: int, tensor_id: int, e: int) -> int:
    return lib().orc_sr_bits(seed, tensor_id, e)


def quantize(T, axis: int, had_block: int, op: Operand, seed: int = 0):
    """-> (codes int8 [lines, D], scale float32, n_eff)."""
    T = _f32(T)
    rows, cols = T.shape
    D = cols if axis else rows
    lines = rows if axis else cols
    codes = np.empty((lines, D), dtype=np.int8)
    scale = C.c_float(0)
    ne = C.c_int(0)
    rc = lib().orc_quantize(_p(T, C.c_float), C.c_int64(rows), C.c_int64(cols), C.c_int(axis),
                            C.c_int(had_block), C.c_int(op.b), C.c_int(op.round_mode),
                            C.c_float(op.clip), C.c_uint32(op.tensor_id), C.c_uint64(seed),
                            _p(codes, C.c_int8), C.byref(scale), C.byref(ne))
    if rc != 0:
        raise ValueError("orc_quantize: bad arguments")
    return codes, np.float32(scale.value), ne.value


def pack_codes(codes, b: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    lines, D = codes.shape
    pitch = lib().orc_packed_pitch(D, b)
    out = np.zeros((lines, pitch), dtype=np.uint8)
    lib().orc_pack_codes(_p(codes, C.c_int8), C.c_int64(lines), C.c_int64(D), C.c_int(b),
                         _p(out, C.c_uint8))
    return out


def tiled_matmul(qA, qB, s: int, a: int) -> np.ndarray:
    qA = np.ascontiguousarray(qA, dtype=np.int8)
    qB = np.ascontiguousarray(qB, dtype=np.int8)
    RA, D = qA.shape
    RB, D2 = qB.shape
    assert D == D2
    acc = np.empty((RA, RB), dtype=np.int32)
    lib().orc_tiled_matmul(_p(qA, C.c_int8), _p(qB, C.c_int8), C.c_int64(RA), C.c_int64(RB),
                           C.c_int64(D), C.c_int64(s), C.c_int(a), _p(acc, C.c_int32))
    return acc


def tiled_matmul_sampled(qA, qB, s: int, a: int, ii, jj) -> np.ndarray:
    qA = np.ascontiguousarray(qA, dtype=np.int8)
    qB = np.ascontiguousarray(qB, dtype=np.int8)
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    D = qA.shape[1]
    assert D == qB.shape[1] and ii.shape == jj.shape
    acc = np.empty(ii.shape[0], dtype=np.int32)
    lib().orc_tiled_matmul_sampled(_p(qA, C.c_int8), _p(qB, C.c_int8), C.c_int64(D),
                                   C.c_int64(s), C.c_int(a), _p(ii, C.c_int64),
                                   _p(jj, C.c_int64), C.c_int64(ii.shape[0]),
                                   _p(acc, C.c_int32))
    return acc


def tiled_matmul_requant(qA, qB, s: int, a: int):
    """Second reading of the accumulator -> (acc int64 [RA, RB], tile_max int32 [tiles]);
    value = acc / 2^(a-1)."""
    qA = np.ascontiguousarray(qA, dtype=np.int8)
    qB = np.ascontiguousarray(qB, dtype=np.int8)
    RA, D = qA.shape
    RB, D2 = qB.shape
    assert D == D2
    tiles = (D + s - 1) // s
    acc = np.empty((RA, RB), dtype=np.int64)
    tmax = np.empty(tiles, dtype=np.int32)
    lib().orc_tiled_matmul_requant(_p(qA, C.c_int8), _p(qB, C.c_int8), C.c_int64(RA), C.c_int64(RB),
                                   C.c_int64(D), C.c_int64(s), C.c_int(a), _p(acc, C.c_int64),
                                   _p(tmax, C.c_int32))
    return acc, tmax


def dequantize_requant(acc, scaleA, scaleB, n: int, a: int) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    out = np.empty(acc.shape, dtype=np.float32)
    lib().orc_dequantize_requant(_p(acc, C.c_int64), C.c_int64(acc.size), C.c_float(scaleA),
                                 C.c_float(scaleB), C.c_int(n), C.c_int(a), _p(out, C.c_float))
    return out


def dequant_factor(scaleA, scaleB, n: int) -> np.float32:
    return np.float32(lib().orc_dequant_factor(C.c_float(scaleA), C.c_float(scaleB), n))


def dequantize(acc, scaleA, scaleB, n: int) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    out = np.empty(acc.shape, dtype=np.float32)
    lib().orc_dequantize(_p(acc, C.c_int32), C.c_int64(acc.size), C.c_float(scaleA),
                         C.c_float(scaleB), C.c_int(n), _p(out, C.c_float))
    return out


def relu_mask(dX, x) -> np.ndarray:
    """dX where x > 0, +0 elsewhere (the rectifier's backward pass applied to an input gradient)."""
    dX = np.ascontiguousarray(dX, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert dX.shape == x.shape
    out = np.empty(dX.shape, dtype=np.float32)
    lib().orc_relu_mask(_p(dX, C.c_float), _p(x, C.c_float), C.c_int64(dX.size), _p(out, C.c_float))
    return out


def bf16_bits(x) -> np.ndarray:
    """binary32 values -> bfloat16 bit patterns (uint16), nearest, ties to even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    f = lib().orc_bf16_bits
    f.restype, f.argtypes = C.c_uint16, [C.c_float]
    return np.array([f(float(v)) for v in x.ravel()], dtype=np.uint16).reshape(x.shape)


def dequantize_bf16(acc, scaleA, scaleB, n: int) -> np.ndarray:
    """Step 6 with the narrow output: uint16 bfloat16 patterns."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    out = np.empty(acc.shape, dtype=np.uint16)
    lib().orc_dequantize_bf16(_p(acc, C.c_int32), C.c_int64(acc.size), C.c_float(scaleA),
                              C.c_float(scaleB), C.c_int(n), _p(out, C.c_uint16))
    return out


def col2im_acc(acc, batch: int, channels: int, H: int, W: int, kh: int, kw: int) -> np.ndarray:
    """Integer accumulators of dX [batch*H*W, C*kh*kw] folded back onto the layer's input:
    int32 [batch, C, H, W] (dequantize() of it is the input gradient)."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    assert acc.shape == (batch * H * W, channels * kh * kw)
    out = np.empty((batch, channels, H, W), dtype=np.int32)
    lib().orc_col2im_acc(_p(acc, C.c_int32), C.c_int64(batch), channels, H, W, kh, kw, _p(out, C.c_int32))
    return out


def gemm_shapes(kind: int, M: int, K: int, N: int):
    """-> (RA, RB, D): output is [RA, RB], contraction length D."""
    return {FWD: (M, N, K), BWD_INPUT: (M, K, N), BWD_WEIGHT: (K, N, M)}[kind]


def gemm(kind: int, P, Q, M: int, K: int, N: int, prm: Params, want_codes: bool = True):
    """One whole matmul.  P, Q are the two source tensors of `kind`:
    FWD (X[M,K], W[K,N]); BWD_INPUT (G[M,N], W[K,N]); BWD_WEIGHT (X[M,K], G[M,N]).
    -> dict(out, acc, codesA, codesB, scaleA, scaleB)."""
    P = _f32(P)
    Q = _f32(Q)
    RA, RB, D = gemm_shapes(kind, M, K, N)
    out = np.empty((RA, RB), dtype=np.float32)
    acc = np.empty((RA, RB), dtype=np.int32)
    cA = np.empty((RA, D), dtype=np.int8) if want_codes else None
    cB = np.empty((RB, D), dtype=np.int8) if want_codes else None
    scales = np.zeros(2, dtype=np.float32)
    c = prm._c()
    rc = lib().orc_gemm(C.c_int(kind), _p(P, C.c_float), _p(Q, C.c_float), C.c_int64(M),
                        C.c_int64(K), C.c_int64(N), C.byref(c), _p(out, C.c_float),
                        _p(acc, C.c_int32),
                        _p(cA, C.c_int8) if want_codes else None,
                        _p(cB, C.c_int8) if want_codes else None,
                        _p(scales, C.c_float))
    if rc != 0:
        raise ValueError("orc_gemm: bad arguments")
    return dict(out=out, acc=acc, codesA=cA, codesB=cB, scaleA=scales[0], scaleB=scales[1])


def num_threads() -> int:
    return int(lib().orc_num_threads())
