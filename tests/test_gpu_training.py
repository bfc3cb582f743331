"""GPU: the forward / backward entry points and the autograd glue on top of them.

hdqt_layer_fwd + hdqt_layer_bwd must reproduce the three per-matmul entry points
bit for bit (those are checked against the oracle elsewhere); the autograd
function must hand autograd exactly what the oracle computes for every matmul of
a small network's training step."""
import numpy as np
import pytest
import torch

from oracle import capi
from paper_2310_03675_amd import autograd as A
from paper_2310_03675_amd import binding as B
from paper_2310_03675_amd import workloads

pytestmark = pytest.mark.gpu

RTOL = 1e-6
FWD, BWI, BWW = B.GEMM_FWD, B.GEMM_BWD_INPUT, B.GEMM_BWD_WEIGHT
O_KIND = {FWD: capi.FWD, BWI: capi.BWD_INPUT, BWW: capi.BWD_WEIGHT}


def dev(t):
    return t.contiguous().to("cuda:0")


def o_params(p: B.Params) -> capi.Params:
    op = lambda o: capi.Operand(b=o.b, round_mode=o.round, clip=o.clip, tensor_id=o.tensor_id)
    return capi.Params(had_block=p.had_block, acc_bits=p.acc_bits, s=p.s, seed=p.seed, A=op(p.A), B=op(p.B))


def assert_matches_oracle(kind, P, Q, M, K, N, prm, got):
    ref = capi.gemm(O_KIND[kind], P.cpu().numpy(), Q.cpu().numpy(), M, K, N, o_params(prm))["out"]
    got = got.detach().cpu().numpy()
    denom = np.maximum(np.abs(ref), np.finfo(np.float32).tiny)
    bad = np.abs(got.astype(np.float64) - ref) > RTOL * denom
    assert not bad.any(), f"kind {kind}: {bad.sum()} of {bad.size} outputs differ"


@pytest.mark.parametrize("M,K,N,n,s,a", [
    (256, 128, 64, 64, 32, 8),
    (512, 1152, 128, 64, 32, 8),
    (128, 561, 561, 64, 32, 8),         # the paper's fully connected width: odd contraction lengths
    (129, 33, 65, 64, 32, 8),
    (4096, 64, 192, 16, 16, 6),
    (64, 64, 64, 8, 1000, 32),
])
def test_layer_fwd_bwd_equals_three_matmuls(M, K, N, n, s, a):
    layer = workloads.fc_layer(M, K, N, seed=5)
    X, W, G = dev(layer.X), dev(layer.W), dev(layer.G)
    cfg = A.LayerConfig(had_block=n, acc_bits=a, s=s, seed=17, layer_id=2)
    pf, pi, pw = (cfg.params(k) for k in (FWD, BWI, BWW))
    print(f"layer_fwd/bwd M={M} K={K} N={N} n={n} s={s} a={a}", flush=True)
    Z, saved = B.layer_fwd(X, W, pf, pw)
    assert saved.numel() == B.load().hdqt_layer_saved_size(M, K, pw.c())
    dX, dW = B.layer_bwd(G, W, saved, K, pi, pw)
    Z3, _, _ = B.gemm(FWD, X, W, M, K, N, pf)
    dX3, _, _ = B.gemm(BWI, G, W, M, K, N, pi)
    dW3, _, _ = B.gemm(BWW, X, G, M, K, N, pw)
    torch.cuda.synchronize()
    assert torch.equal(Z, Z3) and torch.equal(dX, dX3) and torch.equal(dW, dW3)
    # inference (nothing saved) and a first layer (no input gradient)
    Zi, none = B.layer_fwd(X, W, pf, None)
    none_dx, dWb = B.layer_bwd(G, W, saved, K, None, pw)
    torch.cuda.synchronize()
    assert none is None and none_dx is None and torch.equal(Zi, Z3) and torch.equal(dWb, dW3)


@pytest.mark.parametrize("stochastic_act", [False, True])
def test_autograd_three_layer_network_matches_oracle(stochastic_act):
    """Three fully connected layers of width 561 at batch 128 (the paper's continual-
    learning network shape), ReLU between them: every matmul that autograd sees, in
    the forward and in the backward pass, against the oracle on the same operands.
    stochastic_act: the paper's own backward setting, in which the activation of the
    weight-gradient matmul is rounded stochastically as well as the gradient."""
    torch.manual_seed(0)
    widths = [561, 561, 561, 12]
    layers = [A.HdqtLinear(widths[i], widths[i + 1], bias=False,
                           cfg=A.LayerConfig(layer_id=i, seed=3, need_input_grad=(i > 0),
                                             stochastic_act=stochastic_act),
                           device="cuda:0") for i in range(3)]
    x = torch.randn(128, 561, device="cuda:0")
    target = torch.randint(0, 12, (128,), device="cuda:0")
    xs, zs = [], []
    h = x
    for i, layer in enumerate(layers):
        if i > 0:
            h = h.detach().requires_grad_(True)     # cut the graph so each layer's dX is visible
        xs.append(h)
        z = layer(h)
        z.retain_grad()
        zs.append(z)
        h = torch.relu(z)
    loss = torch.nn.functional.cross_entropy(zs[-1], target)
    # backward layer by layer through the cuts
    loss.backward()
    for i in (2, 1):
        g_in = xs[i].grad * (zs[i - 1] > 0)
        zs[i - 1].backward(g_in)
    torch.cuda.synchronize()
    for i, layer in enumerate(layers):
        M, K, N = 128, widths[i], widths[i + 1]
        cfg, W = layer.cfg, layer.weight.detach()
        print(f"layer {i}: {M}x{K}x{N}", flush=True)
        assert_matches_oracle(FWD, xs[i].detach(), W, M, K, N, cfg.params(FWD), zs[i])
        G = zs[i].grad
        assert_matches_oracle(BWW, xs[i].detach(), G, M, K, N, cfg.params(BWW), layer.weight.grad)
        if i > 0:
            assert_matches_oracle(BWI, G, W, M, K, N, cfg.params(BWI), xs[i].grad)
        else:
            assert xs[i].grad is None


def test_training_reduces_the_loss():
    """A few SGD steps of a small quantized network on a synthetic, learnable task: the
    quantized gradients must point downhill (sanity of the glue, not a parity claim)."""
    torch.manual_seed(1)
    net = torch.nn.Sequential(
        A.HdqtLinear(256, 256, cfg=A.LayerConfig(layer_id=0, need_input_grad=False), device="cuda:0"),
        torch.nn.ReLU(),
        A.HdqtLinear(256, 64, cfg=A.LayerConfig(layer_id=1), device="cuda:0"))
    x = torch.randn(512, 256, device="cuda:0")
    teacher = torch.randn(256, 64, device="cuda:0") / 16.0
    y = (x @ teacher).argmax(dim=1)
    opt = torch.optim.SGD(net.parameters(), lr=0.05, momentum=0.9)
    losses = []
    for _ in range(40):
        opt.zero_grad()
        loss = torch.nn.functional.cross_entropy(net(x), y)
        loss.backward()
        opt.step()
        losses.append(loss.item())
    print("loss", losses[0], "->", losses[-1], flush=True)
    assert losses[-1] < 0.5 * losses[0]


def test_conv_block_trains_and_matches_oracle():
    """A small ResNet-style stack (conv 3x3 - ReLU - conv 3x3 - pool - linear) on 16x16
    inputs: the first convolution's three matmuls against the oracle on the operands
    autograd actually passed, and a few SGD steps that must reduce the loss."""
    torch.manual_seed(2)
    conv1 = A.HdqtConv2d(8, 16, cfg=A.LayerConfig(layer_id=0, seed=9), device="cuda:0")
    conv2 = A.HdqtConv2d(16, 32, cfg=A.LayerConfig(layer_id=1, seed=9), device="cuda:0")
    head = A.HdqtLinear(32, 10, cfg=A.LayerConfig(layer_id=2, seed=9), device="cuda:0")
    params = list(conv1.parameters()) + list(conv2.parameters()) + list(head.parameters())
    x = torch.randn(16, 8, 16, 16, device="cuda:0")
    y = torch.randint(0, 10, (16,), device="cuda:0")

    def forward(inp):
        h = torch.relu(conv1(inp))
        h = torch.relu(conv2(h))
        return head(h.mean(dim=(2, 3)))

    # ---- one step with the first convolution's operands captured
    captured = {}
    orig_apply = A.HdqtMatmul.apply

    xin = x.clone().requires_grad_(True)
    cols = torch.nn.functional.unfold(xin, kernel_size=3, padding=1).transpose(1, 2).reshape(16 * 256, 72)
    cols.retain_grad()
    Z = orig_apply(cols, conv1.weight, conv1.cfg, 0)
    Z.retain_grad()
    h = torch.relu(Z.reshape(16, 256, 16).transpose(1, 2).reshape(16, 16, 16, 16))
    h = torch.relu(conv2(h))
    loss = torch.nn.functional.cross_entropy(head(h.mean(dim=(2, 3))), y)
    loss.backward()
    torch.cuda.synchronize()
    M, K, N = 16 * 256, 72, 16
    cfg, W = conv1.cfg, conv1.weight.detach()
    assert_matches_oracle(FWD, cols.detach(), W, M, K, N, cfg.params(FWD, 0), Z)
    assert_matches_oracle(BWW, cols.detach(), Z.grad, M, K, N, cfg.params(BWW, 0), conv1.weight.grad)
    assert_matches_oracle(BWI, Z.grad, W, M, K, N, cfg.params(BWI, 0), cols.grad)

    # ---- a few optimisation steps
    opt = torch.optim.SGD(params, lr=0.05, momentum=0.9)
    losses = []
    for _ in range(60):
        opt.zero_grad()
        loss = torch.nn.functional.cross_entropy(forward(x), y)
        loss.backward()
        opt.step()
        losses.append(loss.item())
    print("loss", losses[0], "->", losses[-1], flush=True)
    assert losses[-1] < 0.85 * losses[0]
