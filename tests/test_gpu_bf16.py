"""GPU parity of the narrow (bfloat16) output of the matmul: hdqt_gemm_codes_bf16 and
hdqt_gemm_bwd_input_bf16 against the oracle's dequantization followed by its bfloat16
rounding.  The 16-bit patterns must be identical: both sides form the same binary32 value
(one multiplication by the same factor) and round it to nearest even."""
import numpy as np
import pytest
import torch

from oracle import capi
from paper_2310_03675_amd import binding as B
from paper_2310_03675_amd import workloads

pytestmark = pytest.mark.gpu


def dev(a):
    t = torch.from_numpy(np.ascontiguousarray(a)) if isinstance(a, np.ndarray) else a
    return t.contiguous().to("cuda:0")


def bits(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def random_codes(rng, lines, D, b, extreme=0.0):
    lo, hi = -(1 << (b - 1)), (1 << (b - 1)) - 1
    c = rng.integers(lo, hi + 1, size=(lines, D)).astype(np.int8)
    if extreme > 0:
        mask = rng.random((lines, D)) < extreme
        c = np.where(mask, np.where(rng.random((lines, D)) < 0.5, lo, hi), c).astype(np.int8)
    return c


# interior tiles with paired stores, edge tiles, odd row lengths (no pairing), a split
# contraction (the second pass narrows), 8-bit codes and ragged tiles (the generic kernel)
@pytest.mark.parametrize("RA,RB,D,bA,bB,s,a", [
    (256, 256, 128, 4, 4, 32, 8),
    (384, 1152, 128, 4, 4, 32, 8),
    (200, 136, 512, 4, 4, 64, 8),
    (130, 129, 256, 4, 4, 32, 8),
    (64, 7, 64, 4, 4, 32, 16),
    (128, 128, 16384, 4, 4, 32, 8),
    (100, 60, 8192 + 64, 4, 4, 64, 8),
    (96, 72, 512, 8, 8, 16, 16),
    (33, 47, 77, 3, 5, 40, 12),
    (1, 1, 64, 4, 4, 32, 8),
])
def test_gemm_codes_bf16(RA, RB, D, bA, bB, s, a):
    print(f"gemm_codes_bf16 RA={RA} RB={RB} D={D} bA={bA} bB={bB} s={s} a={a}", flush=True)
    rng = np.random.default_rng(RA * 7 + RB * 13 + D)
    cA, cB = random_codes(rng, RA, D, bA, 0.2), random_codes(rng, RB, D, bB, 0.2)
    sA, sB, n = np.float32(0.0123), np.float32(3.21e-4), 1
    want_acc = capi.tiled_matmul(cA, cB, s, a)
    want = capi.dequantize_bf16(want_acc, sA, sB, n)
    out, acc = B.gemm_codes(dev(capi.pack_codes(cA, bA)), dev(capi.pack_codes(cB, bB)), bA, bB,
                            dev(np.array([sA])), dev(np.array([sB])), D, n, a, s, bf16=True)
    assert out.dtype == torch.bfloat16
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    got = bits(out)
    assert np.array_equal(got, want), f"{(got != want).sum()} of {got.size} bfloat16 outputs differ"


def test_gemm_codes_bf16_without_accumulators_and_guard_rows():
    """No acc_out; the output buffer is followed by a guard region that must stay untouched."""
    RA, RB, D = 256, 384, 128
    rng = np.random.default_rng(5)
    cA, cB = random_codes(rng, RA, D, 4), random_codes(rng, RB, D, 4)
    one = dev(np.array([1.0], np.float32))
    buf = torch.full((RA + 8, RB), -7.0, dtype=torch.bfloat16, device="cuda:0")
    out = buf[:RA]
    B.gemm_codes(dev(capi.pack_codes(cA, 4)), dev(capi.pack_codes(cB, 4)), 4, 4, one, one, D, 1, 8, 32,
                 want_acc=False, out=out, bf16=True)
    want = capi.dequantize_bf16(capi.tiled_matmul(cA, cB, 32, 8), np.float32(1), np.float32(1), 1)
    assert np.array_equal(bits(out), want)
    assert torch.all(buf[RA:] == -7.0).item()


@pytest.mark.parametrize("M,K,N,n,s", [(64, 256, 128, 16, 16), (512, 1152, 128, 64, 32), (129, 33, 65, 64, 32)])
def test_gemm_bwd_input_bf16(M, K, N, n, s):
    layer = workloads.fc_layer(M, K, N, seed=3)
    prm = B.Params(had_block=n, acc_bits=8, s=s, seed=21,
                   A=B.Operand(4, B.ROUND_STOCHASTIC, 1.0, 6), B=B.Operand(4, B.ROUND_NEAREST, 1.0, 5))
    print(f"gemm_bwd_input_bf16 M={M} K={K} N={N} n={n} s={s}", flush=True)
    out, acc, _ = B.gemm(B.GEMM_BWD_INPUT, dev(layer.G), dev(layer.W), M, K, N, prm, want_acc=True, bf16=True)
    op = lambda o: capi.Operand(b=o.b, round_mode=o.round, clip=o.clip, tensor_id=o.tensor_id)
    ref = capi.gemm(capi.BWD_INPUT, layer.G.numpy(), layer.W.numpy(), M, K, N,
                    capi.Params(had_block=n, acc_bits=8, s=s, seed=21, A=op(prm.A), B=op(prm.B)))
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])
    n_eff = B.n_eff(N, n)
    want = capi.dequantize_bf16(ref["acc"], ref["scaleA"], ref["scaleB"], n_eff)
    assert np.array_equal(bits(out), want)


def test_bwd_input_bf16_resnet_conv_k1152():
    """Full size of the benchmark layer: dX[65536, 1152] in bfloat16.  Sampled positions
    against the oracle (codes quantized in full, sampled accumulators, its narrowing); the
    whole output against the library conversion of the fp32 entry point's result, which
    other tests hold to the oracle."""
    layer = workloads.resnet_conv_layer(256, 128, 128, 16, seed=0)
    M, K, N = layer.M, layer.K, layer.N
    A_op, B_op = B.Operand(4, B.ROUND_STOCHASTIC, 1.0, 6), B.Operand(4, B.ROUND_NEAREST, 1.0, 5)
    prm = B.Params(had_block=64, acc_bits=8, s=32, seed=0, A=A_op, B=B_op)
    G, W = dev(layer.G), dev(layer.W)
    print("bwd_input bf16, 65536 x 1152 x 128", flush=True)
    out16, _, _ = B.gemm(B.GEMM_BWD_INPUT, G, W, M, K, N, prm, bf16=True)
    out32, _, _ = B.gemm(B.GEMM_BWD_INPUT, G, W, M, K, N, prm)
    torch.cuda.synchronize()
    assert torch.equal(out16.view(torch.int16), out32.to(torch.bfloat16).view(torch.int16))
    op = lambda o: capi.Operand(b=o.b, round_mode=o.round, clip=o.clip, tensor_id=o.tensor_id)
    cA, sA, nA = capi.quantize(layer.G.numpy(), 1, 64, op(A_op), 0)
    cB, sB, nB = capi.quantize(layer.W.numpy(), 1, 64, op(B_op), 0)
    rng = np.random.default_rng(8)
    ii, jj = rng.integers(0, M, size=4096), rng.integers(0, K, size=4096)
    ii[:4], jj[:4] = [0, 0, M - 1, M - 1], [0, K - 1, 0, K - 1]
    want = capi.dequantize_bf16(capi.tiled_matmul_sampled(cA, cB, 32, 8, ii, jj), sA, sB, nA)
    got = bits(out16[torch.from_numpy(ii).to("cuda:0"), torch.from_numpy(jj).to("cuda:0")])
    assert np.array_equal(got, want)


def test_bf16_output_rounds_ties_to_even():
    """Totals 257, 259, 261, 263 (and their negatives) with unit scales lie exactly half way
    between two bfloat16 values (8 significant bits): the kernel's conversion must pick
    the even one, like the oracle.  Row i of A times the all-(1) row of B gives the total."""
    D = 256
    totals = [257, 259, 261, 263, -257, -259, 255, 256, 511, 513, 1027]
    cA = np.zeros((128, D), np.int8)
    for i, t in enumerate(totals):
        mag, sign = abs(t), (1 if t > 0 else -1)
        k = 0
        while mag > 0:                      # digits of at most 7 each
            d = min(7, mag)
            cA[i, k] = sign * d
            mag -= d
            k += 1
        assert k <= D
    cB = np.ones((128, D), np.int8)
    one = dev(np.array([1.0], np.float32))
    # 128-row operands with an even row length take the paired-store path; a = 32: nothing saturates
    out, acc = B.gemm_codes(dev(capi.pack_codes(cA, 4)), dev(capi.pack_codes(cB, 4)), 4, 4, one, one,
                            D, 1, 32, 32, bf16=True)
    torch.cuda.synchronize()
    got_acc = acc.cpu().numpy()
    assert [int(v) for v in got_acc[:len(totals), 0]] == totals
    want = capi.dequantize_bf16(got_acc, np.float32(1), np.float32(1), 1)
    assert np.array_equal(bits(out), want)
    as_float = (bits(out).astype(np.uint32) << 16).view(np.float32)
    assert [float(v) for v in as_float[:6, 5]] == [256.0, 260.0, 260.0, 264.0, -256.0, -260.0]
