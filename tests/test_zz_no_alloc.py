"""GPU: hdqt_gemm_fwd_static, the forward matmul for callers that cannot allocate, against
hdqt_gemm_fwd: same outputs and accumulators bit for bit, on two calls in a row through the
library's fixed scratch array, the second on a smaller input (what the first call left in
the array must not be seen)."""
import pytest
import torch

from paper_2310_03675_amd import binding as B
from paper_2310_03675_amd import workloads

pytestmark = pytest.mark.gpu


def _params(n=64, s=32, a=8, seed=5):
    return B.Params(had_block=n, acc_bits=a, s=s, seed=seed,
                    A=B.Operand(4, B.ROUND_NEAREST, 1.0, 0), B=B.Operand(4, B.ROUND_NEAREST, 1.0, 1))


def test_static_forward_matches_workspace_forward_twice():
    prm = _params()
    for M, K, N, scale in ((1024, 1152, 128, 50.0), (320, 192, 72, 1.0)):
        layer = workloads.fc_layer(M, K, N, seed=11)
        # the first call's values are much larger: a calibration maximum left behind would
        # change the second call's scales
        X, W = (layer.X * scale).contiguous().to("cuda:0"), layer.W.contiguous().to("cuda:0")
        print(f"static forward M={M} K={K} N={N}", flush=True)
        Z0, acc0, _ = B.gemm(B.GEMM_FWD, X, W, M, K, N, prm, want_acc=True)
        Z = torch.full((M, N), float("nan"), device="cuda:0")
        acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda:0")
        B.gemm_fwd_static(X, W, prm, Z, acc)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc0)
        assert torch.equal(Z, Z0)
        assert Z.abs().max().item() > 0


def test_static_forward_rejects_what_does_not_fit():
    prm = _params()
    M, K, N = 65536, 1152, 128
    assert B.load().hdqt_workspace_size(B.GEMM_FWD, M, K, N, prm.c()) > B.load().hdqt_gemm_fwd_static_max_bytes()
    X = torch.zeros((M, K), device="cuda:0")
    W = torch.zeros((K, N), device="cuda:0")
    Z = torch.zeros((M, N), device="cuda:0")
    with pytest.raises(B.HdqtError) as err:
        B.gemm_fwd_static(X, W, prm, Z)
    assert err.value.code == -14
