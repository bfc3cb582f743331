"""Pins for the oracle's tiled low-bit-accumulator matmul, dequantization and
the three orientations (paper, Methodology: Z = X W for forward and backward,
tiles of size s; Experiments: 8-bit accumulators, block-size 32)."""
import os

import numpy as np
import pytest
import torch

from oracle import capi, definitional


def _vec(spec, D):
    kind, body = spec.split(":")
    if kind == "c":
        return np.full(D, int(body), dtype=np.int8)
    v = np.array([int(t) for t in body.split(",")], dtype=np.int8)
    assert v.size == D
    return v


def _saturation_cases(golden_dir):
    out = []
    with open(os.path.join(golden_dir, "saturation_cases.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            name, A, B, D, s, a, want = line.split()
            out.append((name, _vec(A, int(D)), _vec(B, int(D)), int(s), int(a), int(want)))
    return out


def test_hand_computed_saturation_cases(golden_dir):
    cases = _saturation_cases(golden_dir)
    assert len(cases) >= 12
    for name, A, B, s, a, want in cases:
        got = capi.tiled_matmul(A[None, :], B[None, :], s, a)
        assert got.shape == (1, 1) and int(got[0, 0]) == want, name
        assert int(definitional.tiled_matmul(A[None, :], B[None, :], s, a)[0, 0]) == want, name
        samp = capi.tiled_matmul_sampled(A[None, :], B[None, :], s, a, [0], [0])
        assert int(samp[0]) == want, name


def test_all_code_pairs_single_element():
    # D = 1: the product of any two 4-bit codes, clamped to the accumulator
    codes = np.arange(-8, 8, dtype=np.int8)[:, None]
    for a in (4, 6, 8):
        got = capi.tiled_matmul(codes, codes, 1, a).astype(np.int64)
        want = np.clip(np.outer(np.arange(-8, 8), np.arange(-8, 8)), -(2 ** (a - 1)), 2 ** (a - 1) - 1)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("s", [1, 5, 16, 32, 1000])
def test_wide_accumulator_is_exact_integer_matmul(s):
    rng = np.random.default_rng(s)
    qA = rng.integers(-8, 8, size=(9, 77), dtype=np.int8)
    qB = rng.integers(-8, 8, size=(13, 77), dtype=np.int8)
    want = qA.astype(np.int64) @ qB.astype(np.int64).T
    assert np.array_equal(capi.tiled_matmul(qA, qB, s, 32).astype(np.int64), want)


def test_no_saturation_means_exact_for_any_tiling():
    # small codes: |tile sum| <= 32*1*7 = 224?  keep it below 127: codes in [-1, 1] x [-3, 3], s <= 32
    rng = np.random.default_rng(1)
    qA = rng.integers(-1, 2, size=(8, 96), dtype=np.int8)
    qB = rng.integers(-3, 4, size=(8, 96), dtype=np.int8)
    want = qA.astype(np.int64) @ qB.astype(np.int64).T
    for s in (7, 16, 32):
        assert np.array_equal(capi.tiled_matmul(qA, qB, s, 8).astype(np.int64), want)


def test_smaller_tiles_saturate_less():
    # the point of tiling: shorter tiles keep partial sums inside the accumulator
    rng = np.random.default_rng(4)
    qA = rng.integers(-8, 8, size=(32, 512), dtype=np.int8)
    qB = rng.integers(-8, 8, size=(32, 512), dtype=np.int8)
    exact = qA.astype(np.int64) @ qB.astype(np.int64).T
    errs = [np.abs(capi.tiled_matmul(qA, qB, s, 8).astype(np.int64) - exact).mean()
            for s in (4, 16, 64, 512)]
    assert errs[0] <= errs[1] <= errs[2] <= errs[3] and errs[3] > errs[0]
    # and a wider accumulator never hurts
    errs_a = [np.abs(capi.tiled_matmul(qA, qB, 32, a).astype(np.int64) - exact).mean()
              for a in (4, 8, 12, 16)]
    assert errs_a[0] >= errs_a[1] >= errs_a[2] >= errs_a[3] == 0


def test_brute_force_against_definitional():
    rng = np.random.default_rng(6)
    for _ in range(25):
        RA, RB, D = (int(v) for v in rng.integers(1, 7, size=3))
        D *= int(rng.choice([1, 3, 8]))
        s = int(rng.integers(1, D + 3))
        a = int(rng.choice([3, 4, 8, 12, 16, 32]))
        qA = rng.integers(-8, 8, size=(RA, D), dtype=np.int8)
        qB = rng.integers(-8, 8, size=(RB, D), dtype=np.int8)
        got = capi.tiled_matmul(qA, qB, s, a).astype(np.int64)
        assert np.array_equal(got, definitional.tiled_matmul(qA, qB, s, a))
        ii = rng.integers(0, RA, size=5)
        jj = rng.integers(0, RB, size=5)
        assert np.array_equal(capi.tiled_matmul_sampled(qA, qB, s, a, ii, jj), got[ii, jj])


def test_dequantize_exact_with_power_of_two_scales():
    acc = np.array([[3, -5], [127, -128]], dtype=np.int32)
    out = capi.dequantize(acc, 0.5, 0.25, 64)
    assert np.array_equal(out, acc.astype(np.float32) * np.float32(0.5 * 0.25 / 64))
    assert capi.dequant_factor(0.5, 0.25, 64) == np.float32(2.0 ** -9)
    assert np.array_equal(definitional.dequantize(acc, 0.5, 0.25, 64), out)


def test_dequantize_rounding_sequence():
    # out = fl(fl(acc) * fl(fl(sA*sB) * 2^-k)): three binary32 roundings in that order
    sA, sB = np.float32(0.1234567), np.float32(7.654321e-3)
    acc = np.array([16777217, -33554435, 1, 12345], dtype=np.int32)   # not all exact in binary32
    dq = np.float32(np.float32(sA * sB) * np.float32(1 / 16))
    want = acc.astype(np.float32) * dq
    assert np.array_equal(capi.dequantize(acc, sA, sB, 16), want)


KINDS = [capi.FWD, capi.BWD_INPUT, capi.BWD_WEIGHT]


def _float_reference(kind, X, W, G):
    X, W, G = (torch.from_numpy(t).double() for t in (X, W, G))
    if kind == capi.FWD:
        return (X @ W).numpy()
    if kind == capi.BWD_INPUT:
        return (G @ W.T).numpy()
    return (X.T @ G).numpy()


def _operands(kind, X, W, G):
    return {capi.FWD: (X, W), capi.BWD_INPUT: (G, W), capi.BWD_WEIGHT: (X, G)}[kind]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("n", [1, 16])
def test_fine_quantization_converges_to_float_matmul(kind, n):
    # b = 8, a = 32: the whole path must approximate the float product; this
    # checks operand choice, contraction axis and transposes of every kind
    rng = np.random.default_rng(10 + kind)
    M, K, N = 48, 64, 32
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) / 8).astype(np.float32)
    G = (rng.standard_normal((M, N)) / 30).astype(np.float32)
    P, Q = _operands(kind, X, W, G)
    prm = capi.Params(had_block=n, acc_bits=32, s=32, A=capi.Operand(b=8), B=capi.Operand(b=8))
    r = capi.gemm(kind, P, Q, M, K, N, prm)
    ref = _float_reference(kind, X, W, G)
    assert r["out"].shape == ref.shape
    rel = np.linalg.norm(r["out"] - ref) / np.linalg.norm(ref)
    assert rel < 2e-2, rel
    # integer accumulators are the exact product of the codes
    want = r["codesA"].astype(np.int64) @ r["codesB"].astype(np.int64).T
    assert np.array_equal(r["acc"].astype(np.int64), want)


@pytest.mark.parametrize("kind", KINDS)
def test_gemm_is_composition_of_its_steps(kind):
    rng = np.random.default_rng(20 + kind)
    M, K, N = 32, 48, 16
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = rng.standard_normal((K, N)).astype(np.float32)
    G = rng.standard_normal((M, N)).astype(np.float32)
    P, Q = _operands(kind, X, W, G)
    axes = {capi.FWD: (1, 0), capi.BWD_INPUT: (1, 1), capi.BWD_WEIGHT: (0, 0)}[kind]
    prm = capi.Params(had_block=16, acc_bits=8, s=16, seed=3,
                      A=capi.Operand(b=4, round_mode=1, tensor_id=1),
                      B=capi.Operand(b=4, tensor_id=2))
    r = capi.gemm(kind, P, Q, M, K, N, prm)
    cA, sA, nA = capi.quantize(P, axes[0], 16, prm.A, seed=3)
    cB, sB, nB = capi.quantize(Q, axes[1], 16, prm.B, seed=3)
    assert nA == nB == 16
    assert np.array_equal(r["codesA"], cA) and np.array_equal(r["codesB"], cB)
    acc = capi.tiled_matmul(cA, cB, 16, 8)
    assert np.array_equal(r["acc"], acc)
    assert np.array_equal(r["out"], capi.dequantize(acc, sA, sB, 16))


def test_hadamard_domain_uses_levels_better_on_outliers():
    # direction check of the paper's histogram figure: with heavy-tailed data,
    # quantizing in the Hadamard domain occupies more of the 16 levels and
    # lowers the error of the product
    from paper_2310_03675_amd import workloads
    X = workloads.outlier_matrix(256, 256, seed=0, role="X").numpy()
    W = workloads.outlier_matrix(256, 256, seed=0, role="W").numpy()
    ref = X.astype(np.float64) @ W.astype(np.float64)
    res = {}
    for n in (1, 64):
        prm = capi.Params(had_block=n, acc_bits=32, s=32, A=capi.Operand(b=4), B=capi.Operand(b=4))
        r = capi.gemm(capi.FWD, X, W, 256, 256, 256, prm)
        hist = np.bincount(r["codesA"].reshape(-1).astype(np.int64) + 8, minlength=16)
        # a level counts as used when it holds at least 0.5 % of the values
        res[n] = (int((hist > 0.005 * hist.sum()).sum()),
                  np.linalg.norm(r["out"] - ref) / np.linalg.norm(ref))
    assert res[64][0] > res[1][0]
    assert res[64][1] < res[1][1]


# ---------------------------------------------------------------- second reading of the accumulator
# (Methodology, tiled quantization: every tile's partial-sum tensor through Q with a bits)

def _codes(rng, rows, D, b=4):
    return rng.integers(-(1 << (b - 1)), 1 << (b - 1), size=(rows, D)).astype(np.int8)


def test_requant_brute_force_against_definitional():
    rng = np.random.default_rng(11)
    for RA, RB, D, s, a in [(5, 4, 12, 4, 8), (3, 6, 20, 8, 5), (4, 4, 7, 3, 3), (2, 2, 64, 32, 8), (6, 3, 9, 100, 12)]:
        qA, qB = _codes(rng, RA, D), _codes(rng, RB, D)
        acc, tmax = capi.tiled_matmul_requant(qA, qB, s, a)
        ref, maxima = definitional.tiled_matmul_requant(qA, qB, s, a)
        assert tmax.tolist() == maxima
        assert acc.tolist() == ref


def test_requant_tile_maxima_are_the_maxima_of_the_integer_products():
    rng = np.random.default_rng(12)
    qA, qB = _codes(rng, 17, 96), _codes(rng, 9, 96)
    _, tmax = capi.tiled_matmul_requant(qA, qB, 32, 8)
    for t in range(3):
        P = qA[:, 32 * t:32 * t + 32].astype(np.int64) @ qB[:, 32 * t:32 * t + 32].astype(np.int64).T
        assert tmax[t] == np.abs(P).max()


def test_requant_with_power_of_two_maxima_is_the_exact_matmul():
    """If every tile's maximum is a power of two not above 2^(a-1) and is reached only by a
    negative partial sum, Q is the identity on that tile (the scale is a power of two, nothing
    rounds, nothing clamps): acc / 2^(a-1) is the plain integer product."""
    rng = np.random.default_rng(13)
    RA, RB, s, tiles, a = 6, 5, 8, 4, 8
    qA = rng.integers(-2, 3, size=(RA, s * tiles)).astype(np.int8)
    qB = rng.integers(-2, 3, size=(RB, s * tiles)).astype(np.int8)
    for t in range(tiles):          # plant the maximum: row 0 x col 0 of each tile sums to -64
        qA[0, s * t:s * t + s] = -8
        qB[0, s * t:s * t + s] = 1
        qA[1:, s * t:s * t + s] = np.clip(qA[1:, s * t:s * t + s], -1, 1)
    acc, tmax = capi.tiled_matmul_requant(qA, qB, s, a)
    P = qA.astype(np.int64) @ qB.astype(np.int64).T
    assert tmax.tolist() == [64] * tiles
    assert np.array_equal(acc, P * 128)


def test_requant_error_is_within_half_a_step_per_tile():
    """|acc / 2^(a-1) - exact| <= sum_t m_t / 2^a, plus one step m_t / 2^(a-1) where the
    positive maximum itself is clamped to 2^(a-1) - 1."""
    rng = np.random.default_rng(14)
    qA, qB = _codes(rng, 40, 256), _codes(rng, 24, 256)
    exact = qA.astype(np.int64) @ qB.astype(np.int64).T
    for s, a in [(32, 8), (64, 6), (16, 4), (256, 8)]:
        acc, tmax = capi.tiled_matmul_requant(qA, qB, s, a)
        err = np.abs(acc / float(1 << (a - 1)) - exact)
        bound = float(np.sum(tmax.astype(np.float64)) / (1 << a) + np.sum(tmax.astype(np.float64)) / (1 << (a - 1)))
        assert err.max() <= bound
        # typical error is far below the bound and shrinks with the accumulator width
        acc_wide, _ = capi.tiled_matmul_requant(qA, qB, s, a + 4)
        assert np.abs(acc_wide / float(1 << (a + 3)) - exact).mean() < err.mean()


def test_requant_single_tile_is_the_quantizer_on_the_product():
    """One tile (s >= D): the reading reduces to Q_a applied to the integer product."""
    rng = np.random.default_rng(15)
    qA, qB = _codes(rng, 12, 48), _codes(rng, 10, 48)
    a = 6
    acc, tmax = capi.tiled_matmul_requant(qA, qB, 1000, a)
    P = qA.astype(np.int64) @ qB.astype(np.int64).T
    m = int(np.abs(P).max())
    assert tmax.tolist() == [m]
    inv = np.float32(np.float64(1 << (a - 1)) / np.float64(m))
    codes = np.clip(np.rint(P.astype(np.float32) * inv), -(1 << (a - 1)), (1 << (a - 1)) - 1).astype(np.int64)
    assert np.array_equal(acc, codes * m)
    # an all-zero operand: every tile's maximum is zero, nothing is added
    acc0, tmax0 = capi.tiled_matmul_requant(np.zeros_like(qA), qB, 16, a)
    assert not acc0.any() and not tmax0.any()


def test_requant_dequantization():
    acc = np.array([[3, -5], [1 << 40, 0]], dtype=np.int64)
    out = capi.dequantize_requant(acc, np.float32(0.5), np.float32(0.25), 64, 8)
    f = np.float32(np.float32(np.float32(0.5) * np.float32(0.25)) * np.float32(1 / 64)) * np.float32(2.0 ** -7)
    assert np.array_equal(out, (acc.astype(np.float32) * f).astype(np.float32))


# ---------------------------------------------------------------- narrow (bfloat16) output

def test_bf16_narrowing_hand_cases():
    """Values whose bfloat16 neighbours are known by construction.  bfloat16 has 7 fraction
    bits, so 1 + 2^-8 is exactly half way between 1 and 1 + 2^-7 and goes to the even one
    (1.0); 1 + 3*2^-8 is half way between 1 + 2^-7 (odd) and 1 + 2^-6 (even) and goes up."""
    cases = [
        (1.0, 0x3F80),
        (1.0 + 2.0 ** -8, 0x3F80),                  # tie, down to even
        (1.0 + 2.0 ** -8 + 2.0 ** -20, 0x3F81),     # just above the tie
        (1.0 + 3 * 2.0 ** -8, 0x3F82),              # tie, up to even
        (1.0 + 2.0 ** -7, 0x3F81),                  # representable
        (-(1.0 + 2.0 ** -8), 0xBF80),               # sign-symmetric
        (2.0 - 2.0 ** -9, 0x4000),                  # rounds up into the next binade
        (0.0, 0x0000),
        (2.0 ** -130, 0x0008),                      # subnormal, representable (2^-133 is the unit)
    ]
    xs = np.array([c[0] for c in cases], dtype=np.float32)
    assert [int(v) for v in capi.bf16_bits(xs)] == [c[1] for c in cases]


def test_bf16_narrowing_against_library_conversion_and_error_bound():
    """Random and adversarial binary32 values against PyTorch's float32 -> bfloat16
    conversion (a library routine for the same IEEE rounding), and the half-unit bound."""
    import torch
    rng = np.random.default_rng(3)
    x = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(1e-3),
        (rng.standard_normal(2000) * 1e4).astype(np.float32),
        # every tie pattern around a few exponents: fraction bits 0x8000 below the cut
        (np.arange(0x3F800000, 0x3F800000 + 256 * 0x10000, 0x8000, dtype=np.uint32)).view(np.float32),
        np.array([3.3895314e38, -3.3895314e38, 1e-40, -1e-40], dtype=np.float32),
    ])
    got = capi.bf16_bits(x)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    back = (got.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    fin = np.isfinite(back)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(x[fin].astype(np.float64)), 2.0 ** -126))) - 7)
    assert np.all(np.abs(back[fin] - x[fin]) <= 0.5 * ulp)


def test_dequantize_bf16_is_narrowing_of_the_fp32_output():
    rng = np.random.default_rng(4)
    acc = rng.integers(-5000, 5000, size=(37, 19)).astype(np.int32)
    sA, sB, n = np.float32(0.0123), np.float32(3.1e-4), 64
    full = capi.dequantize(acc, sA, sB, n)
    assert np.array_equal(capi.dequantize_bf16(acc, sA, sB, n), capi.bf16_bits(full))


# ---------------------------------------------------------------- fold of the input gradient

def _brute_col2im(acc, batch, C, H, W, kh, kw):
    """The transpose of im2col written as a scatter: every entry of dX goes to the input
    element it was read from."""
    out = np.zeros((batch, C, H, W), dtype=np.int64)
    ph, pw = (kh - 1) // 2, (kw - 1) // 2
    for b in range(batch):
        for yp in range(H):
            for xp in range(W):
                m = (b * H + yp) * W + xp
                for c in range(C):
                    for ty in range(kh):
                        for tx in range(kw):
                            y, x = yp + ty - ph, xp + tx - pw
                            if 0 <= y < H and 0 <= x < W:
                                out[b, c, y, x] += acc[m, (c * kh + ty) * kw + tx]
    return out


@pytest.mark.parametrize("batch,C,H,W,kh,kw", [(2, 3, 4, 5, 3, 3), (1, 2, 1, 9, 1, 5), (3, 1, 6, 2, 5, 1),
                                               (2, 2, 3, 3, 1, 1)])
def test_col2im_acc_against_scatter_and_library_fold(batch, C, H, W, kh, kw):
    import torch
    rng = np.random.default_rng(batch * 100 + H * 10 + W)
    acc = rng.integers(-500, 500, size=(batch * H * W, C * kh * kw)).astype(np.int32)
    got = capi.col2im_acc(acc, batch, C, H, W, kh, kw)
    assert np.array_equal(got, _brute_col2im(acc, batch, C, H, W, kh, kw))
    # PyTorch's fold (the adjoint of unfold), exact in float64 on small integers
    cols = torch.from_numpy(acc.astype(np.float64)).reshape(batch, H * W, C * kh * kw).transpose(1, 2)
    ref = torch.nn.functional.fold(cols, output_size=(H, W), kernel_size=(kh, kw),
                                   padding=((kh - 1) // 2, (kw - 1) // 2)).numpy()
    assert np.array_equal(got.astype(np.float64), ref)


def test_col2im_acc_is_the_adjoint_of_im2col():
    """<unfold(a), d> = <a, col2im(d)> for integer tensors: the defining property."""
    import torch
    rng = np.random.default_rng(9)
    batch, C, H, W, kh, kw = 2, 3, 5, 4, 3, 3
    a = rng.integers(-9, 9, size=(batch, C, H, W)).astype(np.float64)
    d = rng.integers(-9, 9, size=(batch * H * W, C * kh * kw)).astype(np.int32)
    X = torch.nn.functional.unfold(torch.from_numpy(a), kernel_size=(kh, kw), padding=1)
    X = X.transpose(1, 2).reshape(batch * H * W, C * kh * kw).numpy()
    lhs = float((X * d).sum())
    rhs = float((a * capi.col2im_acc(d, batch, C, H, W, kh, kw)).sum())
    assert lhs == rhs


def test_col2im_of_a_1x1_window_is_a_transpose():
    rng = np.random.default_rng(10)
    acc = rng.integers(-100, 100, size=(2 * 3 * 4, 5)).astype(np.int32)
    got = capi.col2im_acc(acc, 2, 5, 3, 4, 1, 1)
    assert np.array_equal(got, acc.reshape(2, 12, 5).transpose(0, 2, 1).reshape(2, 5, 3, 4))


# ---------------------------------------------------------------- the rectifier's mask on an input gradient

def test_relu_mask_hand_cases():
    """Written out by hand: kept where the layer's input is positive, +0 elsewhere (also
    where the gradient is negative, where the input is -0, the smallest positive number, or
    negative)."""
    tiny = np.float32(1e-45)            # the smallest positive binary32 (a denormal)
    x = np.array([1.0, -1.0, 0.0, -0.0, tiny, -tiny, 3.5, 2.0], dtype=np.float32)
    dX = np.array([2.5, 2.5, -7.0, 4.0, -3.0, 9.0, -0.0, 1e30], dtype=np.float32)
    want = np.array([2.5, 0.0, 0.0, 0.0, -3.0, 0.0, -0.0, 1e30], dtype=np.float32)
    got = capi.relu_mask(dX, x)
    assert got.tobytes() == want.tobytes()          # bit patterns: masked entries are +0, kept ones untouched


def test_relu_mask_is_the_backward_pass_of_a_rectifier():
    """Against PyTorch's autograd: d/d(pre) of sum(g * max(pre, 0)) is g where max(pre, 0) > 0."""
    import torch
    gen = torch.Generator().manual_seed(3)
    pre = torch.randn((37, 29), generator=gen, requires_grad=True)
    g = torch.randn((37, 29), generator=gen)
    x = torch.relu(pre)
    (x * g).sum().backward()
    got = capi.relu_mask(g.numpy(), x.detach().numpy())
    assert np.array_equal(got, pre.grad.numpy())
    # and it commutes with nothing being masked: an all-positive input leaves the gradient as it is
    assert np.array_equal(capi.relu_mask(g.numpy(), np.ones((37, 29), np.float32)), g.numpy())
