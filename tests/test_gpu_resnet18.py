"""GPU: one training step of a CIFAR-width ResNet-18 at batch 128 whose 21 matmul layers
run through the library (forward, input gradient, weight gradient), followed by an SGD
update.  Images are N(0,1), labels uniform: stand-ins for CIFAR100, which is not
available here.  Parity is per matmul on the operands autograd actually passed: the
step records every layer's X, W, G and its three results, and the oracle recomputes each
product from those exact bits (codes in full, a few thousand sampled outputs).  The glue
between the matmuls (batch norm, ReLU, pooling, unfold / fold) is PyTorch's and is not
under test."""
import numpy as np
import pytest
import torch

from oracle import capi
from paper_2310_03675_amd import binding as B
from paper_2310_03675_amd import resnet, workloads
from paper_2310_03675_amd.autograd import LayerConfig

pytestmark = pytest.mark.gpu

RTOL = 1e-6
SAMPLES = 2048
FWD, BWI, BWW = B.GEMM_FWD, B.GEMM_BWD_INPUT, B.GEMM_BWD_WEIGHT
AXES = {FWD: (1, 0), BWI: (1, 1), BWW: (0, 0)}


def o_op(o):
    return capi.Operand(b=o.b, round_mode=o.round, clip=o.clip, tensor_id=o.tensor_id)


def check_sampled(kind, P, Q, got, prm, rng, cache):
    """Oracle codes of both operands (cached per tensor and axis), then sampled outputs."""
    def codes(role, T, axis, op):
        key = (role, axis, op.round, op.tensor_id)
        if key not in cache:
            cache[key] = capi.quantize(T, axis, prm.had_block, o_op(op), prm.seed)
        return cache[key]
    (roleA, TA), (roleB, TB) = P, Q
    cA, sA, nA = codes(roleA, TA, AXES[kind][0], prm.A)
    cB, sB, nB = codes(roleB, TB, AXES[kind][1], prm.B)
    RA, RB = got.shape
    ii, jj = rng.integers(0, RA, size=SAMPLES), rng.integers(0, RB, size=SAMPLES)
    ii[:4], jj[:4] = [0, 0, RA - 1, RA - 1], [0, RB - 1, 0, RB - 1]
    want_acc = capi.tiled_matmul_sampled(cA, cB, prm.s, prm.acc_bits, ii, jj)
    want = capi.dequantize(want_acc, sA, sB, nA)
    have = got[torch.from_numpy(ii).to(got.device), torch.from_numpy(jj).to(got.device)].cpu().numpy()
    denom = np.maximum(np.abs(want), np.finfo(np.float32).tiny)
    bad = np.abs(have.astype(np.float64) - want) > RTOL * denom
    assert not bad.any(), f"kind {kind}: {bad.sum()} of {bad.size} sampled outputs differ"


def check_fold_sampled(G, W, dAct, shape, kh, prm, rng, cache):
    """The folded input gradient at sampled positions: the oracle's accumulators of the (at most
    kh*kh) entries of dX that fold onto each position, added as integers, dequantized once."""
    batch, C, H, Wd = shape
    def codes(role, T, op):
        key = (role, 1, op.round, op.tensor_id)
        if key not in cache:
            cache[key] = capi.quantize(T, 1, prm.had_block, o_op(op), prm.seed)
        return cache[key]
    cA, sA, nA = codes("G", G, prm.A)
    cB, sB, nB = codes("W", W, prm.B)
    n = 512
    bb, cc = rng.integers(0, batch, n), rng.integers(0, C, n)
    yy, xx = rng.integers(0, H, n), rng.integers(0, Wd, n)
    yy[:4], xx[:4] = [0, 0, H - 1, H - 1], [0, Wd - 1, 0, Wd - 1]
    ph = (kh - 1) // 2
    rows, cols, owner = [], [], []
    for i in range(n):
        for ty in range(kh):
            for tx in range(kh):
                yp, xp = yy[i] - ty + ph, xx[i] - tx + ph
                if 0 <= yp < H and 0 <= xp < Wd:
                    rows.append((bb[i] * H + yp) * Wd + xp)
                    cols.append((cc[i] * kh + ty) * kh + tx)
                    owner.append(i)
    acc = capi.tiled_matmul_sampled(cA, cB, prm.s, prm.acc_bits, np.array(rows), np.array(cols))
    total = np.zeros(n, dtype=np.int64)
    np.add.at(total, np.array(owner), acc.astype(np.int64))
    want = capi.dequantize(total.astype(np.int32), sA, sB, nA)
    idx = [torch.from_numpy(v).to(dAct.device) for v in (bb, cc, yy, xx)]
    have = dAct[idx[0], idx[1], idx[2], idx[3]].cpu().numpy()
    assert np.array_equal(have, want), f"{(have != want).sum()} of {n} folded input gradients differ"


def test_resnet18_training_step_matches_oracle_per_matmul():
    torch.manual_seed(0)
    batch = 128
    cap = {}
    net = resnet.ResNet18(base=LayerConfig(seed=11), device="cuda:0", capture=cap)
    net.train()
    g = torch.Generator().manual_seed(77)
    images = torch.randn((batch, 3, 32, 32), generator=g).to("cuda:0")
    labels = torch.randint(0, 100, (batch,), generator=g).to("cuda:0")
    opt = torch.optim.SGD(net.parameters(), lr=0.05, momentum=0.9, weight_decay=5e-4)
    before = {n: p.detach().clone() for n, p in net.named_parameters()}
    print("forward + backward of ResNet-18, batch 128", flush=True)
    opt.zero_grad()
    loss = torch.nn.functional.cross_entropy(net(images), labels)
    loss.backward()
    opt.step()
    torch.cuda.synchronize()
    assert torch.isfinite(loss).item()
    moved = sum(int(not torch.equal(before[n], p.detach())) for n, p in net.named_parameters())
    assert moved == len(before), "every parameter takes an SGD update"

    table = {name: (M, K, N) for name, M, K, N in workloads.resnet18_layer_table(batch)}
    assert set(cap) == set(table)
    rng = np.random.default_rng(4321)
    fused, folded = [], []
    for name in net.layer_names:
        c = cap[name]
        M, K, N = table[name]
        if "X" not in c:
            # a layer that read its activation directly: the matrix it stands for, by PyTorch's unfold
            kh = {27: 3, 64: 1, 128: 1, 256: 1}.get(K, 3)
            cols = torch.nn.functional.unfold(c["act"].cpu(), kernel_size=kh, padding=kh // 2)
            c["X"] = cols.transpose(1, 2).reshape(M, K).contiguous()
            fused.append(name)
        assert tuple(c["X"].shape) == (M, K) and tuple(c["W"].shape) == (K, N) and tuple(c["G"].shape) == (M, N)
        cfg = LayerConfig(seed=11, layer_id=net.layer_names.index(name))
        print(f"{name}: {M}x{K}x{N}: oracle", flush=True)
        X, W, G = (c[k].cpu().numpy() for k in ("X", "W", "G"))
        cache = {}
        check_sampled(FWD, ("X", X), ("W", W), c["Z"], cfg.params(FWD, c["step"]), rng, cache)
        check_sampled(BWW, ("X", X), ("G", G), c["dW"], cfg.params(BWW, c["step"]), rng, cache)
        if name == "stem":
            assert c["dX"] is None
        elif c.get("dX") is not None:
            check_sampled(BWI, ("G", G), ("W", W), c["dX"], cfg.params(BWI, c["step"]), rng, cache)
        else:
            # the input gradient was folded onto the activation inside the matmul
            check_fold_sampled(G, W, c["dAct"], tuple(c["act"].shape), 3, cfg.params(BWI, c["step"]), rng, cache)
            folded.append(name)
        cap[name] = None            # release the captured tensors of this layer
    # the stride-1 3x3 layers at 32x32, 16x16 and 8x8 read their activation directly
    print("layers that read the activation directly:", fused, flush=True)
    assert len(fused) >= 9
    print("layers whose input gradient was folded inside the matmul:", folded, flush=True)
    assert len(folded) >= 9
