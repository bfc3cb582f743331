"""GPU parity of the folded input gradient: hdqt_gemm_codes_fold / hdqt_conv_bwd write the
gradient of a convolution's input directly; the oracle computes the tiled integer matmul
dX = G W^T on the same codes, folds its accumulators back onto the activation as exact
integer sums and dequantizes once.  The fp32 results must be identical (one multiplication
of the same integer by the same factor on both sides)."""
import numpy as np
import pytest
import torch

from oracle import capi
from paper_2310_03675_amd import binding as B
from paper_2310_03675_amd import workloads

pytestmark = pytest.mark.gpu

NE, ST = B.ROUND_NEAREST, B.ROUND_STOCHASTIC


def dev(a):
    t = torch.from_numpy(np.ascontiguousarray(a)) if isinstance(a, np.ndarray) else a
    return t.contiguous().to("cuda:0")


def random_codes(rng, lines, D, extreme=0.0):
    c = rng.integers(-8, 8, size=(lines, D)).astype(np.int8)
    if extreme > 0:
        mask = rng.random((lines, D)) < extreme
        c = np.where(mask, np.where(rng.random((lines, D)) < 0.5, -8, 7), c).astype(np.int8)
    return c


# (batch, C, H, W, kh, kw, N, s, a): strips with halo rows (32x32; 16x16 with a long contraction), strips without (64 wide, 1 x 3), whole images per
# tile (8x8, 4x4, 2 x 64), a batch that does not fill the last tile, 1-D and 1x1 and 5x5 windows,
# channel counts that are not multiples of the channels per column tile, every epilogue
CASES = [
    (2, 20, 16, 16, 3, 3, 128, 32, 8),
    (1, 14, 32, 32, 3, 3, 64, 32, 8),
    (1, 5, 6, 64, 1, 3, 64, 64, 8),
    (3, 30, 8, 8, 3, 3, 256, 32, 8),
    (5, 9, 4, 4, 3, 3, 64, 32, 8),
    (3, 7, 1, 128, 1, 5, 128, 32, 8),
    (2, 40, 2, 64, 1, 1, 64, 32, 8),
    (2, 6, 16, 8, 5, 5, 64, 64, 8),
    (2, 20, 16, 16, 3, 3, 128, 128, 12),
    (2, 20, 16, 16, 3, 3, 96, 96, 10),
    (1, 3, 40, 16, 3, 1, 32, 32, 6),
    # images of 256 pixels with a contraction of one stage: both halves of an image in one workgroup
    (1, 4, 2, 128, 3, 3, 64, 32, 8),
    (3, 14, 8, 32, 3, 3, 128, 32, 8),
    (2, 15, 32, 8, 3, 3, 128, 64, 8),
    (2, 29, 16, 16, 1, 3, 128, 32, 8),
    (3, 20, 16, 16, 3, 1, 64, 32, 8),
    (2, 20, 16, 16, 3, 3, 160, 32, 8),      # two stages per tile: strips again
    (3, 30, 8, 8, 3, 3, 128, 32, 16),       # wide accumulators whose tiles cannot reach 16 bits
    (2, 20, 16, 16, 3, 3, 128, 128, 15),    # tiles that cannot saturate, merged by the planner
]


@pytest.mark.parametrize("batch,C,H,W,kh,kw,N,s,a", CASES)
def test_gemm_codes_fold(batch, C, H, W, kh, kw, N, s, a):
    M, K = batch * H * W, C * kh * kw
    print(f"fold: act [{batch},{C},{H},{W}] window {kh}x{kw} -> M={M} K={K} N={N} s={s} a={a}", flush=True)
    rng = np.random.default_rng(M + 7 * K + N)
    cG, cW = random_codes(rng, M, N, 0.3), random_codes(rng, K, N, 0.3)
    sG, sW, n = np.float32(0.0123), np.float32(3.21e-4), 32
    acc = capi.tiled_matmul(cG, cW, s, a)
    want = capi.dequantize(capi.col2im_acc(acc, batch, C, H, W, kh, kw), sG, sW, n)
    got = B.gemm_codes_fold(dev(capi.pack_codes(cG, 4)), dev(capi.pack_codes(cW, 4)), 4, 4,
                            dev(np.array([sG])), dev(np.array([sW])), (batch, C, H, W), kh, kw, n, a, s)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert got.shape == want.shape
    bad = got != want
    assert not bad.any(), f"{bad.sum()} of {bad.size} differ, first at {np.argwhere(bad)[0]}"


def test_unsupported_folds_are_refused():
    one = torch.ones(1, device="cuda:0")
    for shape, kh, kw, a, N in (((1, 4, 4, 12), 3, 3, 8, 32),       # width not a power of two
                                ((1, 4, 16, 16), 2, 2, 8, 32),      # even window
                                ((1, 4, 4, 128), 3, 3, 8, 32),      # a strip of one image row cannot hold the halo
                                ((1, 4, 8, 8), 3, 3, 16, 1024)):    # 32 tiles of up to 2048: totals do not fit 16 bits
        b, c, h, w = shape
        qG = torch.zeros((b * h * w, N // 2), dtype=torch.uint8, device="cuda:0")
        qW = torch.zeros((c * kh * kw, N // 2), dtype=torch.uint8, device="cuda:0")
        with pytest.raises(B.HdqtError) as e:
            B.gemm_codes_fold(qG, qW, 4, 4, one, one, shape, kh, kw, 32, a, 32)
        assert e.value.code == -13, (shape, kh, kw, a, e.value.code)


def test_conv_bwd_matches_layer_bwd_and_library_fold():
    """hdqt_conv_fwd + hdqt_conv_bwd on a layer: dW identical to hdqt_layer_bwd's; dAct against
    the oracle (integer fold of the oracle's own accumulators), and close to PyTorch's fold of
    the fp32 gradient of the im2col matrix (same sum, rounded term by term instead of once)."""
    torch.manual_seed(3)
    batch, C, H, W, N = 4, 64, 16, 16, 128
    act = torch.relu(torch.randn(batch, C, H, W))
    K, M = C * 9, batch * H * W
    g = torch.Generator().manual_seed(5)
    Wt = torch.randn((K, N), generator=g) * (2.0 / K) ** 0.5
    G = torch.randn((M, N), generator=g) * 1e-2
    mk = lambda A, Bq: B.Params(had_block=64, acc_bits=8, s=32, seed=7, A=A, B=Bq)
    pf = mk(B.Operand(4, NE, 1.0, 0), B.Operand(4, NE, 1.0, 1))
    pi = mk(B.Operand(4, ST, 1.0, 6), B.Operand(4, NE, 1.0, 5))
    pw = mk(B.Operand(4, NE, 1.0, 8), B.Operand(4, ST, 1.0, 10))
    Z, saved = B.conv_fwd(dev(act), 3, 3, dev(Wt), pf, pw)
    dAct, dW = B.conv_bwd(dev(G), dev(Wt), saved, (batch, C, H, W), 3, 3, pi, pw)
    dXcol, dW2 = B.layer_bwd(dev(G), dev(Wt), saved, K, pi, pw)
    torch.cuda.synchronize()
    assert torch.equal(dW, dW2)
    op = lambda o: capi.Operand(b=o.b, round_mode=o.round, clip=o.clip, tensor_id=o.tensor_id)
    ref = capi.gemm(capi.BWD_INPUT, G.numpy(), Wt.numpy(), M, K, N,
                    capi.Params(had_block=64, acc_bits=8, s=32, seed=7, A=op(pi.A), B=op(pi.B)))
    want = capi.dequantize(capi.col2im_acc(ref["acc"], batch, C, H, W, 3, 3), ref["scaleA"], ref["scaleB"], 64)
    assert np.array_equal(dAct.cpu().numpy(), want)
    folded = torch.nn.functional.fold(dXcol.reshape(batch, H * W, K).transpose(1, 2), output_size=(H, W),
                                      kernel_size=3, padding=1)
    # (term-by-term rounding against one rounding: absolute error of a few ulps of the largest term)
    assert torch.allclose(dAct, folded, rtol=1e-5, atol=9 * 2.0 ** -22 * float(dXcol.abs().max()))
