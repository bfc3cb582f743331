"""GPU parity of the input gradient behind a rectifier: hdqt_gemm_bwd_input_masked,
hdqt_layer_bwd_masked and hdqt_conv_bwd_masked write dX (or the folded dAct) where the layer's
input is positive and +0 elsewhere.  The oracle computes the whole matmul from the fp32
tensors and applies orc_relu_mask to its result."""
import numpy as np
import pytest
import torch

from oracle import capi
from paper_2310_03675_amd import autograd as A
from paper_2310_03675_amd import binding as B
from paper_2310_03675_amd import workloads

pytestmark = pytest.mark.gpu

RTOL = 1e-6
NE, ST = B.ROUND_NEAREST, B.ROUND_STOCHASTIC
BWI = B.GEMM_BWD_INPUT


def dev(t):
    return t.contiguous().to("cuda:0")


def params(n, s, a, b=4, seed=9):
    return B.Params(had_block=n, acc_bits=a, s=s, seed=seed, A=B.Operand(b, ST, 1.0, 6), B=B.Operand(b, NE, 1.0, 5))


def o_params(p):
    op = lambda o: capi.Operand(b=o.b, round_mode=o.round, clip=o.clip, tensor_id=o.tensor_id)
    return capi.Params(had_block=p.had_block, acc_bits=p.acc_bits, s=p.s, seed=p.seed, A=op(p.A), B=op(p.B))


def assert_masked(got, want_unmasked, x):
    want = capi.relu_mask(want_unmasked, x)
    keep = x > 0
    assert np.all(got[~keep].view(np.uint32) == 0), "masked entries must be +0"
    denom = np.maximum(np.abs(want), np.finfo(np.float32).tiny)
    assert np.all(np.abs(got.astype(np.float64) - want) <= RTOL * denom)
    assert keep.any() and (~keep).any() and np.count_nonzero(want) > 0


# the matrix-core kernel's own masked epilogue (8-bit tiles of 32 and 64, whole-stage tiles, the
# generic clamp), a narrow output, a contraction split over workgroups (masked by the pass that
# adds the slices), byte codes and the generic kernel (masked by a pass of their own)
@pytest.mark.parametrize("M,K,N,n,s,a,b", [
    (512, 256, 128, 64, 32, 8, 4),
    (384, 200, 192, 64, 64, 8, 4),
    (256, 128, 256, 64, 128, 16, 4),
    (300, 130, 96, 32, 96, 10, 4),
    (1024, 48, 64, 64, 32, 8, 4),
    (128, 128, 8192, 64, 32, 8, 4),
    (512, 256, 128, 64, 32, 16, 8),
    (129, 33, 65, 64, 32, 8, 4),
    (64, 27, 100, 64, 7, 6, 3),
])
def test_gemm_bwd_input_masked(M, K, N, n, s, a, b):
    layer = workloads.fc_layer(M, K, N, seed=21)
    X = torch.relu(layer.X - 0.3)            # a rectifier's output: about 40 % positive, the rest +0
    X[0, 0] = -0.0 if K else 0.0
    prm = params(n, s, a, b)
    print(f"masked bwd_input M={M} K={K} N={N} n={n} s={s} a={a} b={b}", flush=True)
    out, acc, _ = B.gemm(BWI, dev(layer.G), dev(layer.W), M, K, N, prm, want_acc=True, mask=dev(X))
    plain, acc0, _ = B.gemm(BWI, dev(layer.G), dev(layer.W), M, K, N, prm, want_acc=True)
    torch.cuda.synchronize()
    ref = capi.gemm(capi.BWD_INPUT, layer.G.numpy(), layer.W.numpy(), M, K, N, o_params(prm))
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])            # the accumulators are not masked
    assert_masked(out.cpu().numpy(), ref["out"], X.numpy())
    assert torch.equal(out, torch.where(dev(X) > 0, plain, torch.zeros_like(plain)))


def test_gemm_bwd_input_masked_resnet_conv_k1152():
    """The benchmark layer's input gradient (302 MB, streamed stores) with the mask of its own
    input: sampled against the oracle, and in full against the unmasked call."""
    layer = workloads.resnet_conv_layer(256, 128, 128, 16, seed=0)
    M, K, N = layer.M, layer.K, layer.N
    prm = params(64, 32, 8, seed=0)
    G, W, X = dev(layer.G), dev(layer.W), dev(layer.X)
    out, _, ws = B.gemm(BWI, G, W, M, K, N, prm, mask=X)
    plain, _, _ = B.gemm(BWI, G, W, M, K, N, prm, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out, torch.where(X > 0, plain, torch.zeros_like(plain)))
    print("oracle quantization ...", flush=True)
    cA, sA, nA = capi.quantize(layer.G.numpy(), 1, 64, o_params(prm).A, 0)
    cB, sB, _ = capi.quantize(layer.W.numpy(), 1, 64, o_params(prm).B, 0)
    rng = np.random.default_rng(5)
    ii, jj = rng.integers(0, M, 4096), rng.integers(0, K, 4096)
    want = capi.dequantize(capi.tiled_matmul_sampled(cA, cB, 32, 8, ii, jj), sA, sB, nA)
    x = layer.X.numpy()[ii, jj]
    got = out[torch.from_numpy(ii).to("cuda:0"), torch.from_numpy(jj).to("cuda:0")].cpu().numpy()
    assert_masked(got, want, x)


@pytest.mark.parametrize("M,K,N", [(512, 256, 128), (128, 561, 561), (129, 33, 65)])
def test_layer_bwd_masked(M, K, N):
    layer = workloads.fc_layer(M, K, N, seed=4)
    X = torch.relu(layer.X)
    cfg = A.LayerConfig(seed=3, layer_id=1)
    pf, pi, pw = (cfg.params(k) for k in (B.GEMM_FWD, BWI, B.GEMM_BWD_WEIGHT))
    Xd, Wd, Gd = dev(X), dev(layer.W), dev(layer.G)
    _, saved = B.layer_fwd(Xd, Wd, pf, pw)
    dX, dW = B.layer_bwd(Gd, Wd, saved, K, pi, pw, mask=Xd)
    dX0, dW0 = B.layer_bwd(Gd, Wd, saved, K, pi, pw)
    torch.cuda.synchronize()
    assert torch.equal(dW, dW0)
    ref = capi.gemm(capi.BWD_INPUT, layer.G.numpy(), layer.W.numpy(), M, K, N, o_params(pi))["out"]
    assert_masked(dX.cpu().numpy(), ref, X.numpy())


@pytest.mark.parametrize("batch,C,H,W,N", [(2, 64, 16, 16, 64), (2, 64, 8, 8, 128), (1, 64, 32, 32, 64)])
def test_conv_bwd_masked(batch, C, H, W, N):
    """The folded input gradient behind a rectifier: the mask is the activation itself."""
    gen = torch.Generator().manual_seed(batch + C)
    act = torch.relu(torch.randn((batch, C, H, W), generator=gen))
    M, K = batch * H * W, C * 9
    Wt = torch.randn((K, N), generator=gen) * (2.0 / K) ** 0.5
    G = torch.randn((M, N), generator=gen) * 1e-2
    cfg = A.LayerConfig(seed=2, layer_id=3)
    pf, pi, pw = (cfg.params(k) for k in (B.GEMM_FWD, BWI, B.GEMM_BWD_WEIGHT))
    act_d, W_d, G_d = dev(act), dev(Wt), dev(G)
    _, saved = B.conv_fwd(act_d, 3, 3, W_d, pf, pw)
    dAct, dW = B.conv_bwd(G_d, W_d, saved, (batch, C, H, W), 3, 3, pi, pw, mask=act_d)
    dAct0, dW0 = B.conv_bwd(G_d, W_d, saved, (batch, C, H, W), 3, 3, pi, pw)
    torch.cuda.synchronize()
    assert torch.equal(dW, dW0)
    # oracle: the matmul's accumulators folded back as integers, dequantized once, then the mask
    o = o_params(pi)
    cG, sG, n = capi.quantize(G.numpy(), 1, pi.had_block, o.A, pi.seed)
    cW, sW, _ = capi.quantize(Wt.numpy(), 1, pi.had_block, o.B, pi.seed)
    acc = capi.tiled_matmul(cG, cW, pi.s, pi.acc_bits)
    want = capi.dequantize(capi.col2im_acc(acc, batch, C, H, W, 3, 3), sG, sW, n)
    assert_masked(dAct.cpu().numpy(), want, act.numpy())
    assert torch.equal(dAct, torch.where(act_d > 0, dAct0, torch.zeros_like(dAct0)))


def test_relu_linear_module_matches_separate_rectifier():
    """HdqtLinear(relu_input=True) against relu followed by HdqtLinear: same output, same weight
    gradient, same gradient of the rectifier's input."""
    torch.manual_seed(0)
    cfg = A.LayerConfig(seed=5, layer_id=0)
    fused = A.HdqtLinear(192, 96, bias=False, cfg=cfg, device="cuda:0", relu_input=True)
    plain = A.HdqtLinear(192, 96, bias=False, cfg=cfg, device="cuda:0")
    with torch.no_grad():
        plain.weight.copy_(fused.weight)
    pre1 = torch.randn(256, 192, device="cuda:0", requires_grad=True)
    pre2 = pre1.detach().clone().requires_grad_(True)
    g = torch.randn(256, 96, device="cuda:0") * 1e-2
    z1 = fused(pre1)
    z2 = plain(torch.relu(pre2))
    z1.backward(g)
    z2.backward(g)
    torch.cuda.synchronize()
    assert torch.equal(z1, z2) and torch.equal(fused.weight.grad, plain.weight.grad)
    assert torch.equal(pre1.grad, pre2.grad)
