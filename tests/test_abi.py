"""The C-ABI library loads, exports every symbol include/hdqt.h declares, and
rejects bad arguments on the host before anything is launched (no GPU needed:
no call here reaches a kernel launch)."""
import ctypes as C
import os
import re

import pytest

from paper_2310_03675_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = C.c_void_p(0x10000)          # non-null, 16-byte aligned, never dereferenced on the host


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "hdqt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hdqt_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = B.load()
    names = _declared_functions()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTED) == names


def test_block_order_and_pitch_helpers():
    assert B.n_eff(576, 64) == 64 and B.n_eff(1152, 64) == 64 and B.n_eff(27, 64) == 1
    assert B.n_eff(100, 64) == 4 and B.n_eff(320, 32) == 32 and B.n_eff(96, 64) == 32
    assert B.codes_pitch(27, 4) == 14 and B.codes_pitch(27, 8) == 27 and B.codes_pitch(64, 3) == 32


def test_struct_layout_matches_header():
    assert C.sizeof(B.COperand) == 16
    assert C.sizeof(B.CParams) == 8 + 8 + 8 + 32
    assert B.CParams.s.offset == 8 and B.CParams.seed.offset == 16 and B.CParams.A.offset == 24


def test_workspace_layout():
    p = B.Params(had_block=64, acc_bits=8, s=32)
    L = B.workspace_layout(B.GEMM_BWD_WEIGHT, 65536, 1152, 128, p)
    assert (L.RA, L.RB, L.D, L.n_eff) == (1152, 128, 65536, 64)
    assert L.codesA % 256 == 0 and L.codesB % 256 == 0 and L.acc % 256 == 0
    assert L.codesB - L.codesA >= 1152 * 32768
    assert L.total >= L.acc + 1152 * 128 * 4
    assert B.workspace_size(B.GEMM_BWD_WEIGHT, 65536, 1152, 128, p) == L.total
    L = B.workspace_layout(B.GEMM_FWD, 128, 27, 64, p)
    assert (L.RA, L.RB, L.D, L.n_eff) == (128, 64, 27, 1)
    L = B.workspace_layout(B.GEMM_BWD_INPUT, 128, 512, 100, p)
    assert (L.RA, L.RB, L.D, L.n_eff) == (128, 512, 100, 4)


def _gemm_rc(kind=B.GEMM_FWD, M=64, K=64, N=64, ws_bytes=1 << 20, **over):
    p = B.Params(**{k: v for k, v in over.items() if k in ("had_block", "acc_bits", "s")})
    if "A" in over:
        p.A = over["A"]
    if "B" in over:
        p.B = over["B"]
    cp = p.c()
    fn = getattr(B.load(), B._GEMM_FN[kind])
    return fn(over.get("P", FAKE), over.get("Q", FAKE), over.get("out", FAKE), M, K, N,
              C.byref(cp), None, over.get("ws", FAKE), ws_bytes, None)


@pytest.mark.parametrize("kind", [B.GEMM_FWD, B.GEMM_BWD_INPUT, B.GEMM_BWD_WEIGHT])
def test_gemm_argument_errors(kind):
    assert _gemm_rc(kind, P=None) == -1
    assert _gemm_rc(kind, out=None) == -1
    assert _gemm_rc(kind, M=0) == -2
    assert _gemm_rc(kind, N=-5) == -2
    assert _gemm_rc(kind, K=1 << 31) == -2
    assert _gemm_rc(kind, had_block=48) == -3
    assert _gemm_rc(kind, had_block=512) == -3
    assert _gemm_rc(kind, had_block=0) == -3
    assert _gemm_rc(kind, A=B.Operand(b=1)) == -4
    assert _gemm_rc(kind, B=B.Operand(b=9)) == -4
    assert _gemm_rc(kind, acc_bits=1) == -5
    assert _gemm_rc(kind, acc_bits=33) == -5
    assert _gemm_rc(kind, s=0) == -6
    assert _gemm_rc(kind, A=B.Operand(clip=0.0)) == -7
    assert _gemm_rc(kind, A=B.Operand(clip=1.5)) == -7
    assert _gemm_rc(kind, B=B.Operand(round=2)) == -8
    assert _gemm_rc(kind, ws=None) == -10
    assert _gemm_rc(kind, ws_bytes=16) == -10
    assert _gemm_rc(kind, P=C.c_void_p(0x10004)) == -11


def test_accumulation_range_errors():
    # 8-bit codes, one tile of 2^20: tile sum up to 2^34 does not fit int32
    big = dict(A=B.Operand(b=8), B=B.Operand(b=8))
    assert _gemm_rc(B.GEMM_FWD, M=64, K=1 << 20, N=64, s=1 << 20, acc_bits=32, ws_bytes=1 << 40, **big) == -6
    # about 2^22 tiles of one element, each up to 2^14: total up to 2^36
    assert _gemm_rc(B.GEMM_FWD, M=16, K=65535 * 64, N=16, s=1, acc_bits=16, ws_bytes=1 << 40, **big) == -5


def test_unknown_kind():
    p = B.Params().c()
    assert B.load().hdqt_workspace_layout(7, 8, 8, 8, C.byref(p), None) == -9
    assert B.load().hdqt_workspace_size(7, 8, 8, 8, C.byref(p)) == 0


def _quant_rc(T=FAKE, rows=64, cols=64, axis=1, had=64, op=None, codes=FAKE, scale=FAKE, ws=FAKE,
              ws_bytes=1 << 16):
    cop = (op or B.Operand()).c()
    return B.load().hdqt_quantize(T, rows, cols, axis, had, C.byref(cop), 0, codes, scale, ws,
                                  ws_bytes, None)


def test_quantize_argument_errors():
    assert _quant_rc(T=None) == -1
    assert _quant_rc(codes=None) == -1
    assert _quant_rc(scale=None) == -1
    assert _quant_rc(rows=0) == -2
    assert _quant_rc(axis=2) == -9
    assert _quant_rc(had=3) == -3
    assert _quant_rc(op=B.Operand(b=0)) == -4
    assert _quant_rc(op=B.Operand(clip=-1.0)) == -7
    assert _quant_rc(op=B.Operand(round=5)) == -8
    assert _quant_rc(ws=None) == -10
    assert _quant_rc(ws_bytes=8) == -10
    assert _quant_rc(T=C.c_void_p(0x10008)) == -11


def test_gemm_codes_argument_errors():
    lib = B.load()

    def rc(qA=FAKE, qB=FAKE, bA=4, bB=4, sA=FAKE, sB=FAKE, RA=8, RB=8, D=64, n=64, a=8, s=32,
           out=FAKE, acc=None):
        return lib.hdqt_gemm_codes(qA, qB, bA, bB, sA, sB, RA, RB, D, n, a, s, out, acc, None, 0,
                                   None)
    assert rc(qA=None) == -1
    assert rc(out=None, acc=None) == -1
    assert rc(RA=0) == -2
    assert rc(bA=9) == -4
    assert rc(n=48) == -3
    assert rc(D=96, n=64) == -3
    assert rc(a=40) == -5
    assert rc(s=0) == -6


def test_strerror_texts():
    assert B.strerror(0) == "success"
    for code in range(-13, 0):
        assert B.strerror(code) and "unknown error" not in B.strerror(code)
    assert "unknown error" in B.strerror(-99)
    assert B.load().hdqt_last_hip_error() == 0


# ---------------------------------------------------------------- the whole-step entry points
# (argument errors only: found on the host before anything is launched)

def _error_codes():
    """name -> value of the HDQT_E* macros, parsed from the header"""
    text = open(os.path.join(ROOT, "include", "hdqt.h")).read()
    return {k: int(v) for k, v in re.findall(r"#define (HDQT_E[A-Z_]+) \((-\d+)\)", text)}


E = _error_codes()


def _cparams(n=64, a=8, s=32, bA=4, bB=4):
    return B.Params(had_block=n, acc_bits=a, s=s, A=B.Operand(b=bA), B=B.Operand(b=bB)).c()


def test_quantize_dual_argument_errors():
    lib = B.load()
    op = B.Operand(b=4).c()

    def rc(T=FAKE, rows=64, cols=64, had=64, o1=op, o0=op, c1=FAKE, s1=FAKE, c0=FAKE, s0=FAKE,
           ws=FAKE, ws_bytes=1 << 16):
        return lib.hdqt_quantize_dual(T, rows, cols, had, C.byref(o1), C.byref(o0), 0, c1, s1, c0, s0,
                                      ws, ws_bytes, None)

    assert lib.hdqt_quantize_dual_workspace_size() >= 2 * lib.hdqt_quantize_workspace_size()
    assert rc(T=None) == E["HDQT_EINVAL_NULL"]
    assert rc(c0=None) == E["HDQT_EINVAL_NULL"]
    assert rc(s1=None) == E["HDQT_EINVAL_NULL"]
    assert rc(rows=0) == E["HDQT_EINVAL_DIM"]
    assert rc(had=48) == E["HDQT_EINVAL_HADAMARD"]
    assert rc(o0=B.Operand(b=9).c()) == E["HDQT_EINVAL_BITS"]
    assert rc(o1=B.Operand(b=4, clip=0.0).c()) == E["HDQT_EINVAL_CLIP"]
    assert rc(ws=None) == E["HDQT_EWORKSPACE"]
    assert rc(ws_bytes=lib.hdqt_quantize_workspace_size()) == E["HDQT_EWORKSPACE"]
    assert rc(c1=C.c_void_p(0x1008)) == E["HDQT_EALIGN"]
    assert rc(s0=C.c_void_p(0x1002)) == E["HDQT_EALIGN"]


def test_layer_step_argument_errors():
    lib = B.load()
    M, K, N = 256, 128, 64
    pf, pi, pw = _cparams(), _cparams(), _cparams()
    need = lib.hdqt_layer_step_workspace_size(M, K, N, C.byref(pf), C.byref(pi), C.byref(pw))
    assert need > 0
    # without the input gradient less is needed, never more
    assert 0 < lib.hdqt_layer_step_workspace_size(M, K, N, C.byref(pf), None, C.byref(pw)) <= need
    assert lib.hdqt_layer_step_workspace_size(M, K, N, C.byref(pf), C.byref(pi), C.byref(_cparams(n=3))) == 0

    def rc(X=FAKE, W=FAKE, G=FAKE, Z=FAKE, dX=FAKE, dW=FAKE, m=M, f=pf, i=pi, w=pw, ws=FAKE, nbytes=need):
        return lib.hdqt_layer_step(X, W, G, Z, dX, dW, m, K, N, C.byref(f) if f else None,
                                   C.byref(i) if i else None, C.byref(w) if w else None, ws, nbytes, None)

    assert rc(X=None) == E["HDQT_EINVAL_NULL"]
    assert rc(dW=None) == E["HDQT_EINVAL_NULL"]
    assert rc(w=None) == E["HDQT_EINVAL_NULL"]
    assert rc(i=None) == E["HDQT_EINVAL_NULL"]            # dX wanted but no parameters for it
    assert rc(m=0) == E["HDQT_EINVAL_DIM"]
    assert rc(f=_cparams(a=1)) == E["HDQT_EINVAL_ACC"]
    assert rc(w=_cparams(s=0)) == E["HDQT_EINVAL_TILE"]
    assert rc(i=_cparams(bA=1)) == E["HDQT_EINVAL_BITS"]
    assert rc(ws=None) == E["HDQT_EWORKSPACE"]
    assert rc(nbytes=need - 1) == E["HDQT_EWORKSPACE"]
    assert rc(G=C.c_void_p(0x1004)) == E["HDQT_EALIGN"]


def test_layer_fwd_bwd_argument_errors():
    lib = B.load()
    M, K, N = 256, 128, 64
    pf, pi, pw = _cparams(), _cparams(), _cparams()
    saved = lib.hdqt_layer_saved_size(M, K, C.byref(pw))
    assert saved >= K * M // 2 and lib.hdqt_layer_saved_size(M, K, None) == 0
    nf = lib.hdqt_layer_fwd_workspace_size(M, K, N, C.byref(pf), C.byref(pw))
    nb = lib.hdqt_layer_bwd_workspace_size(M, K, N, C.byref(pi), C.byref(pw))
    assert nf > 0 and nb > 0
    assert lib.hdqt_layer_bwd_workspace_size(M, K, N, C.byref(pi), None) == 0

    def fwd(X=FAKE, W=FAKE, Z=FAKE, f=pf, w=pw, sv=FAKE, sv_bytes=saved, ws=FAKE, nbytes=nf):
        return lib.hdqt_layer_fwd(X, W, Z, M, K, N, C.byref(f) if f else None, C.byref(w) if w else None,
                                  sv, sv_bytes, ws, nbytes, None)

    assert fwd(Z=None) == E["HDQT_EINVAL_NULL"]
    assert fwd(f=None) == E["HDQT_EINVAL_NULL"]
    assert fwd(sv=None) == E["HDQT_EINVAL_NULL"]          # codes are to be saved but there is no buffer
    assert fwd(sv_bytes=saved - 1) == E["HDQT_EWORKSPACE"]
    assert fwd(nbytes=nf - 1) == E["HDQT_EWORKSPACE"]
    assert fwd(f=_cparams(n=512)) == E["HDQT_EINVAL_HADAMARD"]
    assert fwd(sv=C.c_void_p(0x1001)) == E["HDQT_EALIGN"]

    def bwd(G=FAKE, W=FAKE, sv=FAKE, dX=FAKE, dW=FAKE, i=pi, w=pw, ws=FAKE, nbytes=nb):
        return lib.hdqt_layer_bwd(G, W, sv, dX, dW, M, K, N, C.byref(i) if i else None,
                                  C.byref(w) if w else None, ws, nbytes, None)

    assert bwd(G=None) == E["HDQT_EINVAL_NULL"]
    assert bwd(sv=None) == E["HDQT_EINVAL_NULL"]
    assert bwd(w=None) == E["HDQT_EINVAL_NULL"]
    assert bwd(i=None) == E["HDQT_EINVAL_NULL"]
    assert bwd(W=None) == E["HDQT_EINVAL_NULL"]
    assert bwd(nbytes=nb - 1) == E["HDQT_EWORKSPACE"]
    assert bwd(w=_cparams(a=40)) == E["HDQT_EINVAL_ACC"]
    assert bwd(dW=C.c_void_p(0x1008)) == E["HDQT_EALIGN"]


def test_gemm_codes_workspace_size():
    lib = B.load()
    assert lib.hdqt_gemm_codes_workspace_size(65536, 128, 1152, 32) == 0          # many output tiles: no split
    need = lib.hdqt_gemm_codes_workspace_size(1152, 128, 65536, 32)               # 9 tiles, long contraction
    assert need > 0 and need % (1152 * 128 * 4) == 0
    assert lib.hdqt_gemm_codes_workspace_size(0, 128, 64, 32) == 0


def test_gemm_codes_requant_argument_errors():
    lib = B.load()
    assert lib.hdqt_gemm_codes_requant_workspace_size(8, 8, 64, 32) >= 2 * 8 * 8 * 4 + 2 * 4
    assert lib.hdqt_gemm_codes_requant_workspace_size(8, 0, 64, 32) == 0
    # the exact size for given widths: no tile sums where the two-pass path runs, the bound elsewhere
    assert 0 < lib.hdqt_gemm_codes_requant_workspace_size_for(8, 8, 64, 32, 4, 4, 8) < 2 * 8 * 8 * 4
    assert lib.hdqt_gemm_codes_requant_workspace_size_for(8, 8, 64, 32, 8, 8, 8) == \
        lib.hdqt_gemm_codes_requant_workspace_size(8, 8, 64, 32)
    assert lib.hdqt_gemm_codes_requant_workspace_size_for(8, 8, 64, 32, 4, 4, 40) == 0
    assert lib.hdqt_gemm_codes_requant_workspace_size_for(8, 8, 64, 32, 9, 4, 8) == 0

    def rc(qA=FAKE, bA=4, bB=4, RA=8, D=64, n=64, a=8, s=32, out=FAKE, ws=FAKE, nbytes=1 << 20):
        return lib.hdqt_gemm_codes_requant(qA, FAKE, bA, bB, FAKE, FAKE, RA, 8, D, n, a, s, out, None, ws,
                                           nbytes, None)

    assert rc(qA=None) == E["HDQT_EINVAL_NULL"]
    assert rc(out=None) == E["HDQT_EINVAL_NULL"]
    assert rc(RA=0) == E["HDQT_EINVAL_DIM"]
    assert rc(bA=1) == E["HDQT_EINVAL_BITS"]
    assert rc(n=3) == E["HDQT_EINVAL_HADAMARD"]
    assert rc(a=25) == E["HDQT_EINVAL_ACC"]
    assert rc(s=0) == E["HDQT_EINVAL_TILE"]
    assert rc(bA=8, bB=8, D=4096, s=4096) == E["HDQT_EINVAL_TILE"]     # 4096 * 2^14 = 2^26: not exact in binary32
    assert rc(D=1 << 20, n=64, a=16) == E["HDQT_EINVAL_ACC"]           # the sum over 32768 tiles may leave int32
    assert rc(ws=None) == E["HDQT_EWORKSPACE"]
    assert rc(nbytes=64) == E["HDQT_EWORKSPACE"]
    p = _cparams()
    assert lib.hdqt_gemm_requant_workspace_size(0, 256, 128, 64, C.byref(p)) > 0
    assert lib.hdqt_gemm_requant_workspace_size(5, 256, 128, 64, C.byref(p)) == 0
    assert lib.hdqt_gemm_requant(0, None, FAKE, FAKE, 256, 128, 64, C.byref(p), None, FAKE, 1 << 30, None) \
        == E["HDQT_EINVAL_NULL"]
    assert lib.hdqt_gemm_requant(0, FAKE, FAKE, FAKE, 256, 128, 64, C.byref(p), None, FAKE, 1024, None) \
        == E["HDQT_EWORKSPACE"]


def test_dimension_limit():
    """A dimension above 65535 * 64 is refused: the grids could not hold it."""
    p = _cparams()
    lim = 65535 * 64
    assert B.load().hdqt_workspace_size(0, lim, 64, 64, C.byref(p)) > 0
    assert B.load().hdqt_workspace_size(0, lim + 1, 64, 64, C.byref(p)) == 0
    assert _quant_rc(rows=lim + 1) == E["HDQT_EINVAL_DIM"]
    assert _quant_rc(cols=lim + 64, had=64) == E["HDQT_EINVAL_DIM"]


def test_bf16_output_argument_errors():
    """The narrow-output entry points check their arguments like the fp32 ones."""
    lib = B.load()

    def rc(qA=FAKE, bA=4, RA=8, D=64, n=64, a=8, s=32, out=FAKE, acc=None):
        return lib.hdqt_gemm_codes_bf16(qA, FAKE, bA, 4, FAKE, FAKE, RA, 8, D, n, a, s, out, acc, None, 0,
                                        None)
    assert rc(qA=None) == E["HDQT_EINVAL_NULL"]
    assert rc(out=None, acc=None) == E["HDQT_EINVAL_NULL"]
    assert rc(RA=0) == E["HDQT_EINVAL_DIM"]
    assert rc(bA=9) == E["HDQT_EINVAL_BITS"]
    assert rc(n=48) == E["HDQT_EINVAL_HADAMARD"]
    assert rc(a=40) == E["HDQT_EINVAL_ACC"]
    assert rc(s=0) == E["HDQT_EINVAL_TILE"]
    assert rc(out=C.c_void_p(0x10002)) == E["HDQT_EALIGN"]
    p = _cparams()
    f = lib.hdqt_gemm_bwd_input_bf16
    assert f(None, FAKE, FAKE, 64, 64, 64, C.byref(p), None, FAKE, 1 << 30, None) == E["HDQT_EINVAL_NULL"]
    assert f(FAKE, FAKE, None, 64, 64, 64, C.byref(p), None, FAKE, 1 << 30, None) == E["HDQT_EINVAL_NULL"]
    assert f(FAKE, FAKE, FAKE, 64, 64, 64, C.byref(p), None, FAKE, 16, None) == E["HDQT_EWORKSPACE"]
    assert f(FAKE, FAKE, FAKE, 0, 64, 64, C.byref(p), None, FAKE, 1 << 30, None) == E["HDQT_EINVAL_DIM"]


def test_conv_source_argument_errors():
    """hdqt_quantize_dual_im2col / hdqt_conv_step: geometry and argument errors are found on
    the host."""
    lib = B.load()
    op = B.Operand(b=4).c()
    good = B.CConv(2, 64, 16, 16, 3, 3)

    def rc(act=FAKE, geo=good, n=64, ws=FAKE, ws_bytes=1 << 20):
        return lib.hdqt_quantize_dual_im2col(act, C.byref(geo) if geo is not None else None, n, C.byref(op),
                                             C.byref(op), 0, FAKE, FAKE, FAKE, FAKE, ws, ws_bytes, None)
    assert rc(act=None) == E["HDQT_EINVAL_NULL"]
    assert rc(geo=None) == E["HDQT_EINVAL_NULL"]
    assert rc(geo=B.CConv(0, 64, 16, 16, 3, 3)) == E["HDQT_EINVAL_DIM"]
    assert rc(n=48) == E["HDQT_EINVAL_HADAMARD"]
    assert rc(ws_bytes=8) == E["HDQT_EWORKSPACE"]
    for bad in (B.CConv(2, 64, 16, 16, 2, 2), B.CConv(2, 64, 12, 12, 3, 3), B.CConv(2, 3, 16, 16, 3, 3),
                B.CConv(2, 64, 3, 16, 3, 3), B.CConv(1, 64, 8, 8, 1, 1)):
        assert rc(geo=bad) == E["HDQT_EINVAL_GEOMETRY"]
    p = _cparams()
    size = lib.hdqt_conv_step_workspace_size
    assert size(C.byref(good), 128, C.byref(p), C.byref(p), C.byref(p)) == \
        lib.hdqt_layer_step_workspace_size(512, 576, 128, C.byref(p), C.byref(p), C.byref(p)) > 0
    assert size(C.byref(B.CConv(2, 64, 12, 12, 3, 3)), 128, C.byref(p), C.byref(p), C.byref(p)) == 0
    step = lib.hdqt_conv_step
    args = lambda geo, dx=FAKE: (FAKE, C.byref(geo), FAKE, FAKE, FAKE, dx, FAKE, 128, C.byref(p), C.byref(p),
                                 C.byref(p), FAKE, 1 << 30, None)
    assert step(*args(good, dx=None)) == E["HDQT_EINVAL_NULL"]
    assert step(*args(B.CConv(2, 64, 12, 12, 3, 3))) == E["HDQT_EINVAL_GEOMETRY"]
    assert step(*args(B.CConv(2, 64, 16, 16, 3, 3))[:-3], FAKE, 16, None) == E["HDQT_EWORKSPACE"]


def test_folded_input_gradient_argument_errors():
    lib = B.load()
    good = B.CConv(2, 64, 16, 16, 3, 3)

    def rc(qG=FAKE, geo=good, N=128, n=64, a=8, s=32, out=FAKE, bG=4):
        return lib.hdqt_gemm_codes_fold(qG, FAKE, bG, 4, FAKE, FAKE, C.byref(geo) if geo is not None else None,
                                        N, n, a, s, out, None)
    assert rc(qG=None) == E["HDQT_EINVAL_NULL"]
    assert rc(out=None) == E["HDQT_EINVAL_NULL"]
    assert rc(geo=None) == E["HDQT_EINVAL_NULL"]
    assert rc(N=0) == E["HDQT_EINVAL_DIM"]
    assert rc(n=48) == E["HDQT_EINVAL_HADAMARD"]
    assert rc(a=40) == E["HDQT_EINVAL_ACC"]
    assert rc(out=C.c_void_p(0x10004)) == E["HDQT_EALIGN"]
    # geometries and settings the fold does not take: refused before anything is launched
    assert rc(geo=B.CConv(2, 64, 12, 12, 3, 3)) == E["HDQT_EINVAL_GEOMETRY"]
    assert rc(geo=B.CConv(2, 64, 16, 16, 2, 2)) == E["HDQT_EINVAL_GEOMETRY"]
    assert rc(geo=B.CConv(2, 64, 4, 128, 3, 3)) == E["HDQT_EINVAL_GEOMETRY"]
    assert rc(a=16, N=1024) == E["HDQT_EINVAL_GEOMETRY"]   # 32 tiles of up to 2048: totals beyond 16 bits
    assert rc(bG=8) == E["HDQT_EINVAL_GEOMETRY"]           # 8-bit codes: not the 4-bit kernel
    assert rc(s=48) == E["HDQT_EINVAL_GEOMETRY"]           # tile length not a multiple of 32
    p = _cparams()
    f = lib.hdqt_conv_bwd
    args = lambda geo=good, dact=FAKE, ws=1 << 30: (FAKE, FAKE, FAKE, C.byref(geo), dact, FAKE, 128, C.byref(p),
                                                   C.byref(p), FAKE, ws, None)
    assert f(*args(dact=None)) == E["HDQT_EINVAL_NULL"]
    assert f(*args(geo=B.CConv(2, 64, 12, 12, 3, 3))) == E["HDQT_EINVAL_GEOMETRY"]
    assert f(*args(ws=16)) == E["HDQT_EWORKSPACE"]


def test_im2col_argument_errors():
    f = B.load().hdqt_im2col
    ok = (FAKE, 2, 3, 8, 8, 3, 3, 1, 1, 1, FAKE, None)
    bad = lambda i, v: f(*(ok[:i] + (v,) + ok[i + 1:]))
    assert bad(0, None) == E["HDQT_EINVAL_NULL"] and bad(10, None) == E["HDQT_EINVAL_NULL"]
    assert bad(1, 0) == E["HDQT_EINVAL_DIM"]          # batch
    assert bad(7, 0) == E["HDQT_EINVAL_DIM"]          # stride
    assert bad(5, 12) == E["HDQT_EINVAL_DIM"]         # window taller than the padded image
    assert bad(8, -1) == E["HDQT_EINVAL_DIM"]         # negative padding
    assert bad(10, C.c_void_p(0x10008)) == E["HDQT_EALIGN"]
