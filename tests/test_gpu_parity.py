"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on the same seeded inputs.  Integer outputs (codes, accumulators)
must be bit-exact; dequantized fp32 outputs within 1e-6 relative."""
import numpy as np
import pytest
import torch

from oracle import capi
from paper_2310_03675_amd import binding as B
from paper_2310_03675_amd import workloads

pytestmark = pytest.mark.gpu

RTOL = 1e-6


def dev(a):
    t = torch.from_numpy(np.ascontiguousarray(a)) if isinstance(a, np.ndarray) else a
    return t.contiguous().to("cuda:0")


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def assert_close_f32(got, want):
    assert got.shape == want.shape
    denom = np.maximum(np.abs(want), np.finfo(np.float32).tiny)
    bad = np.abs(got.astype(np.float64) - want.astype(np.float64)) > RTOL * denom
    assert not bad.any(), f"{bad.sum()} of {bad.size} outputs differ by more than {RTOL} relative"


def o_operand(op: B.Operand) -> capi.Operand:
    return capi.Operand(b=op.b, round_mode=op.round, clip=op.clip, tensor_id=op.tensor_id)


def o_params(p: B.Params) -> capi.Params:
    return capi.Params(had_block=p.had_block, acc_bits=p.acc_bits, s=p.s, seed=p.seed,
                       A=o_operand(p.A), B=o_operand(p.B))


# ------------------------------------------------------------------ quantize

def check_quantize(T: np.ndarray, axis: int, n: int, op: B.Operand, seed: int = 0):
    print(f"quantize shape={T.shape} axis={axis} n={n} b={op.b} round={op.round} clip={op.clip}",
          flush=True)
    codes_g, scale_g = B.quantize(dev(T), axis, n, op, seed)
    codes_o, scale_o, n_eff = capi.quantize(T, axis, n, o_operand(op), seed)
    want = capi.pack_codes(codes_o, op.b)
    got = host(codes_g)
    assert got.shape == want.shape
    assert host(scale_g)[0] == scale_o, (host(scale_g)[0], scale_o)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"{len(bad)} code bytes differ, first at {bad[0]}: "
                             f"got {got[tuple(bad[0])]:#x} want {want[tuple(bad[0])]:#x}")
    assert B.n_eff(T.shape[1] if axis == 1 else T.shape[0], n) == n_eff


QUANT_SHAPES = [
    # (rows, cols, axis, n)
    (64, 256, 1, 16), (256, 128, 0, 16), (64, 128, 1, 16), (64, 128, 0, 16),   # FC layer operands
    (33, 320, 1, 32), (320, 40, 0, 32), (320, 40, 0, 64),
    (70, 576, 1, 64), (576, 24, 0, 64), (1152, 36, 0, 64),
    (8, 512, 1, 256), (1024, 40, 0, 256), (512, 12, 0, 128), (16, 1024, 1, 128),
    (3, 100, 1, 64), (100, 7, 0, 64), (5, 27, 1, 64), (27, 5, 0, 64),          # n_eff 4, 1 (odd D)
    (64, 101, 0, 64), (7, 6, 1, 8), (6, 7, 0, 8), (1, 8, 1, 8), (8, 1, 0, 8),
    (300, 96, 0, 64), (2048, 48, 0, 64), (48, 2048, 1, 64), (520, 33, 0, 8),
    (129, 64, 1, 1), (64, 129, 0, 1),
    # axis 0, block orders 128 and 256: whole strips, a strip that ends early, ragged column strips
    (384, 36, 0, 128), (768, 132, 0, 256), (256, 64, 0, 256), (1280, 32, 0, 256), (640, 68, 0, 128),
    (2304, 260, 0, 256),
]


@pytest.mark.parametrize("rows,cols,axis,n", QUANT_SHAPES)
def test_quantize_nearest_4bit(rows, cols, axis, n):
    rng = np.random.default_rng(rows * 1000 + cols)
    T = (rng.standard_normal((rows, cols)) * 3.0).astype(np.float32)
    check_quantize(T, axis, n, B.Operand(b=4))


@pytest.mark.parametrize("rows,cols,axis,n", QUANT_SHAPES)
def test_quantize_stochastic_4bit(rows, cols, axis, n):
    rng = np.random.default_rng(rows * 1000 + cols + 1)
    T = (rng.standard_normal((rows, cols)) * 1e-2).astype(np.float32)
    check_quantize(T, axis, n, B.Operand(b=4, round=B.ROUND_STOCHASTIC, tensor_id=7), seed=0x1234567887654321)


@pytest.mark.parametrize("b", [2, 3, 5, 6, 8])
@pytest.mark.parametrize("rows,cols,axis,n", [(40, 192, 1, 64), (192, 40, 0, 64), (9, 27, 1, 64),
                                              (27, 9, 0, 64), (3, 100, 1, 4), (512, 40, 0, 256),
                                              (384, 36, 0, 128)])
def test_quantize_other_widths(b, rows, cols, axis, n):
    rng = np.random.default_rng(b * 77 + rows)
    T = rng.standard_normal((rows, cols)).astype(np.float32)
    check_quantize(T, axis, n, B.Operand(b=b, clip=0.975))
    check_quantize(T, axis, n, B.Operand(b=b, round=B.ROUND_STOCHASTIC, tensor_id=b), seed=b)


def test_quantize_degenerate_inputs():
    check_quantize(np.zeros((16, 64), np.float32), 1, 64, B.Operand(b=4))
    check_quantize(np.zeros((64, 16), np.float32), 0, 64, B.Operand(b=4, round=B.ROUND_STOCHASTIC))
    one = np.zeros((64, 64), np.float32)
    one[5, 9] = -3.0
    check_quantize(one, 1, 64, B.Operand(b=4))
    check_quantize(one, 0, 64, B.Operand(b=4))
    # ties and exact grid values
    grid = (np.arange(-64, 64, dtype=np.float32) / 8.0).reshape(2, 64)
    grid[0, 0] = 8.0
    check_quantize(grid, 1, 1, B.Operand(b=4))
    check_quantize(grid, 1, 1, B.Operand(b=4, round=B.ROUND_STOCHASTIC, tensor_id=3), seed=9)


def test_quantize_heavy_tails_and_wide_range():
    X = workloads.outlier_matrix(512, 256, seed=0, role="X").numpy()
    for n in (64, 256):
        check_quantize(X, 1, n, B.Operand(b=4))
        check_quantize(X, 0, n, B.Operand(b=4))
    rng = np.random.default_rng(5)
    T = (rng.standard_normal((256, 256)) * 10.0 ** rng.integers(-6, 6, size=(256, 256))).astype(np.float32)
    check_quantize(T, 1, 64, B.Operand(b=8))
    check_quantize(T, 0, 64, B.Operand(b=8))


# ------------------------------------------------------------------ integer matmul on codes

def random_codes(rng, lines, D, b, extreme=0.0):
    lo, hi = -(1 << (b - 1)), (1 << (b - 1)) - 1
    c = rng.integers(lo, hi + 1, size=(lines, D)).astype(np.int8)
    if extreme > 0:
        mask = rng.random((lines, D)) < extreme
        c = np.where(mask, np.where(rng.random((lines, D)) < 0.5, lo, hi), c).astype(np.int8)
    return c


def check_gemm_codes(RA, RB, D, bA, bB, s, a, n=1, extreme=0.0, seed=0):
    print(f"gemm_codes RA={RA} RB={RB} D={D} bA={bA} bB={bB} s={s} a={a}", flush=True)
    rng = np.random.default_rng(seed + RA * 7 + RB * 13 + D)
    cA = random_codes(rng, RA, D, bA, extreme)
    cB = random_codes(rng, RB, D, bB, extreme)
    sA, sB = np.float32(0.0123), np.float32(3.21e-4)
    want_acc = capi.tiled_matmul(cA, cB, s, a)
    want_out = capi.dequantize(want_acc, sA, sB, n)
    out, acc = B.gemm_codes(dev(capi.pack_codes(cA, bA)), dev(capi.pack_codes(cB, bB)), bA, bB,
                            dev(np.array([sA])), dev(np.array([sB])), D, n, a, s)
    got_acc, got_out = host(acc), host(out)
    if not np.array_equal(got_acc, want_acc):
        bad = np.argwhere(got_acc != want_acc)
        raise AssertionError(f"{len(bad)} accumulators differ, first at {bad[0]}: got "
                             f"{got_acc[tuple(bad[0])]} want {want_acc[tuple(bad[0])]}")
    assert_close_f32(got_out, want_out)


@pytest.mark.parametrize("s", [16, 32, 64, 256])
@pytest.mark.parametrize("a", [8, 16, 32])
def test_gemm_codes_aligned(s, a):
    check_gemm_codes(200, 136, 512, 4, 4, s, a, n=64)
    check_gemm_codes(200, 136, 512, 4, 4, s, a, n=64, extreme=0.5)


@pytest.mark.parametrize("s", [1, 5, 16, 27, 32, 48, 100, 1000])
def test_gemm_codes_ragged(s):
    check_gemm_codes(37, 29, 100, 4, 4, s, 8, n=4, extreme=0.3)
    check_gemm_codes(130, 5, 27, 4, 4, s, 8, extreme=0.3)
    check_gemm_codes(9, 300, 144, 4, 4, s, 6, n=16, extreme=0.3)


@pytest.mark.parametrize("bA,bB", [(8, 8), (4, 8), (3, 5), (2, 2), (8, 4)])
def test_gemm_codes_widths(bA, bB):
    for s, a in ((16, 8), (64, 16), (40, 12), (512, 32)):
        check_gemm_codes(96, 72, 512, bA, bB, s, a, n=64, extreme=0.2)
        check_gemm_codes(33, 47, 77, bA, bB, s, a, n=1, extreme=0.2)


@pytest.mark.parametrize("bA,bB", [(8, 8), (5, 6), (6, 8), (7, 5)])
def test_gemm_codes_byte_codes_matrix_path(bA, bB):
    """Both operands with a byte per code, tiles that are multiples of 32: the matrix-core
    kernel's instances for unpacked codes (whole stages when 128 divides s)."""
    for s, a in ((32, 8), (32, 12), (64, 16), (96, 32), (128, 12), (128, 32), (256, 16), (384, 32)):
        check_gemm_codes(200, 136, 768, bA, bB, s, a, n=64, extreme=0.3)
    check_gemm_codes(128, 256, 64, bA, bB, 32, 12, n=64, extreme=0.2)      # one short stage
    check_gemm_codes(1, 1, 4096, bA, bB, 32, 10, n=64, extreme=0.9)
    # all codes at the negative end: the largest tile sums there are
    D = 256
    cA = np.full((130, D), -(1 << (bA - 1)), np.int8)
    cB = np.full((70, D), -(1 << (bB - 1)), np.int8)
    one = dev(np.array([1.0], np.float32))
    for s, a in ((32, 32), (128, 32), (64, 16)):
        out, acc = B.gemm_codes(dev(capi.pack_codes(cA, bA)), dev(capi.pack_codes(cB, bB)), bA, bB, one, one,
                                D, 1, a, s)
        assert np.array_equal(host(acc), capi.tiled_matmul(cA, cB, s, a))


@pytest.mark.parametrize("bA,bB,accs", [
    (4, 4, (9, 10, 11, 12, 13, 16)), (3, 4, (8, 9, 12)), (2, 3, (8, 10)), (4, 2, (11,)),
    (5, 5, (10, 12, 14, 16)), (5, 6, (11, 12, 13)), (6, 6, (12, 15)), (7, 8, (15, 16)), (8, 8, (16,)),
    (8, 5, (13, 14)),
])
def test_gemm_codes_saturation_through_int16(bA, bB, accs):
    """Accumulators of bA + bB to 16 bits with tiles of 32 and 64: the operands are scaled on
    their way to LDS so that the int16 conversion is the clamp.  Half the codes sit at the
    ends of their range, so most tile sums saturate."""
    for a in accs:
        for s in (16, 32, 64):
            check_gemm_codes(200, 136, 768, bA, bB, s, a, n=64, extreme=0.5)
            check_gemm_codes(130, 70, 64, bA, bB, s, a, n=64, extreme=0.9)
            check_gemm_codes(96, 40, 96, bA, bB, s, a, n=32, extreme=0.05)
    # every code at the negative end, every code at the positive end, and mixed signs
    D = 256
    lo = lambda b: -(1 << (b - 1))
    hi = lambda b: (1 << (b - 1)) - 1
    one = dev(np.array([1.0], np.float32))
    for va, vb in ((lo(bA), lo(bB)), (hi(bA), hi(bB)), (lo(bA), hi(bB)), (hi(bA), lo(bB))):
        cA = np.full((64, D), va, np.int8)
        cB = np.full((64, D), vb, np.int8)
        for s in (16, 32, 64):
            out, acc = B.gemm_codes(dev(capi.pack_codes(cA, bA)), dev(capi.pack_codes(cB, bB)), bA, bB,
                                    one, one, D, 1, accs[0], s)
            assert np.array_equal(host(acc), capi.tiled_matmul(cA, cB, s, accs[0])), (va, vb, s)


@pytest.mark.parametrize("D", [40, 72, 216, 1144, 4104])
def test_gemm_codes_rows_that_end_inside_a_step(D):
    """Contraction lengths that are multiples of 8 (packed codes) or 4 (a byte per code) but
    not of 32: the matrix-core kernel takes them and clears, on the way to LDS, what the last
    16-byte unit of a row read from the next row.  Half the codes at the range ends, so that
    a code leaking in from the next row would change a saturating tile."""
    for s, a in ((32, 8), (64, 8), (16, 8), (32, 12), (96, 32), (128, 16), (256, 16)):
        if s > D and s != 32:
            continue
        check_gemm_codes(200, 136, D, 4, 4, s, a, n=8, extreme=0.5)
    check_gemm_codes(130, 40, D, 4, 4, 32, 8, n=8, extreme=0.5)           # the 128 x 64 tile
    check_gemm_codes(200, 136, D + 4, 8, 8, 32, 16, n=4, extreme=0.5)     # bytes: a multiple of 4
    check_gemm_codes(200, 136, D + 12, 6, 7, 64, 32, n=4, extreme=0.5)
    check_requant_codes(200, 136, D, 4, 4, 32, 8, n=8, extreme=0.3)


def test_gemm_codes_rows_that_end_inside_a_step_split_contraction():
    check_gemm_codes(128, 128, 65544, 4, 4, 32, 8, n=8, extreme=0.3)      # 2049 tiles, split into parts
    check_gemm_codes(256, 64, 32776, 4, 4, 64, 8, n=8, extreme=0.3)


@pytest.mark.parametrize("RA,RB", [(300, 64), (128, 33), (1000, 1), (50, 60), (513, 64)])
def test_gemm_codes_outputs_of_at_most_64_columns(RA, RB):
    """The 128 x 64 workgroup tile: every epilogue that has such instances, ragged rows and
    columns, one stage and many, a split contraction."""
    for s, a in ((32, 8), (64, 8), (128, 8), (256, 16), (96, 6), (32, 32), (64, 7)):
        check_gemm_codes(RA, RB, 768, 4, 4, s, a, n=64, extreme=0.4)
    check_gemm_codes(RA, RB, 64, 4, 3, 32, 8, n=64, extreme=0.9)
    check_gemm_codes(RA, RB, 16384 + 96, 4, 4, 32, 8, n=32, extreme=0.3)


def test_gemm_codes_tiles_of_16_codes():
    """Two tiles per 32-code step of the matrix-core kernel, 8-bit and wider accumulators,
    split contractions whose parts would start in the middle of a step."""
    for a in (8, 9, 11):
        check_gemm_codes(200, 136, 768, 4, 4, 16, a, n=16, extreme=0.4)
        check_gemm_codes(70, 130, 32, 4, 4, 16, a, n=16, extreme=0.9)
    check_gemm_codes(200, 136, 768, 3, 3, 16, 8, n=16, extreme=0.4)
    check_gemm_codes(128, 128, 16384, 4, 4, 16, 8, n=64, extreme=0.4)
    check_gemm_codes(64, 64, 4096 + 32, 4, 4, 16, 9, n=32, extreme=0.5)
    check_gemm_codes(100, 60, 8192 + 64, 8, 8, 16, 16, n=64, extreme=0.5)
    check_gemm_codes(64, 64, 16 * 31 * 8 + 32, 5, 5, 16, 12, n=32, extreme=0.5)
    # accumulators narrower than bA + bB bits: the compare-select clamp on the same loop
    for bA, bB, a in ((4, 4, 6), (4, 3, 5), (8, 8, 8), (5, 8, 10), (8, 8, 12)):
        check_gemm_codes(200, 136, 768, bA, bB, 16, a, n=16, extreme=0.4)
        check_gemm_codes(70, 130, 32, bA, bB, 16, a, n=16, extreme=0.9)
    check_gemm_codes(128, 128, 16384, 8, 8, 16, 8, n=64, extreme=0.4)
    check_gemm_codes(64, 64, 4096 + 32, 4, 4, 16, 6, n=32, extreme=0.5)


def test_gemm_codes_saturation_through_int16_split_contraction():
    check_gemm_codes(128, 128, 16384, 4, 4, 32, 12, n=64, extreme=0.6)
    check_gemm_codes(100, 60, 8192 + 64, 8, 8, 64, 16, n=64, extreme=0.5)
    check_gemm_codes(64, 64, 4096 + 32, 5, 6, 32, 11, n=32, extreme=0.5)


def test_gemm_codes_byte_codes_split_contraction():
    check_gemm_codes(128, 128, 16384, 8, 8, 32, 12, n=64, extreme=0.1)
    check_gemm_codes(100, 60, 8192 + 64, 8, 6, 128, 16, n=64, extreme=0.5)
    check_gemm_codes(64, 64, 4096, 5, 8, 64, 32, n=64, extreme=0.5)


def test_gemm_codes_split_contraction():
    # few output tiles and a long contraction: several workgroups share a tile
    check_gemm_codes(128, 128, 16384, 4, 4, 32, 8, n=64, extreme=0.1)
    check_gemm_codes(100, 60, 8192 + 64, 4, 4, 64, 8, n=64, extreme=0.5)
    check_gemm_codes(64, 64, 4096, 4, 4, 48, 8, n=64, extreme=0.5)
    check_gemm_codes(1, 1, 4096, 4, 4, 16, 4, n=64, extreme=0.9)


def gaussian_codes(rng, lines, D, sigma):
    return np.clip(np.rint(rng.normal(0.0, sigma, size=(lines, D))), -8, 7).astype(np.int8)


def check_gemm_codes_given(cA, cB, s, a):
    D = cA.shape[1]
    n = 64 if D % 64 == 0 else 8
    print(f"gemm_codes (given codes) RA={cA.shape[0]} RB={cB.shape[0]} D={D} s={s} a={a}", flush=True)
    want_acc = capi.tiled_matmul(cA, cB, s, a)
    one = dev(np.array([1.0], np.float32))
    out, acc = B.gemm_codes(dev(capi.pack_codes(cA, 4)), dev(capi.pack_codes(cB, 4)), 4, 4, one, one, D, n, a, s)
    got_acc = host(acc)
    if not np.array_equal(got_acc, want_acc):
        bad = np.argwhere(got_acc != want_acc)
        raise AssertionError(f"{len(bad)} accumulators differ, first at {bad[0]}: got "
                             f"{got_acc[tuple(bad[0])]} want {want_acc[tuple(bad[0])]}")
    assert_close_f32(host(out), capi.dequantize(want_acc, np.float32(1.0), np.float32(1.0), n))


@pytest.mark.parametrize("RA,RB,D", [(384, 256, 1152), (300, 64, 576), (256, 128, 16384), (130, 200, 1144)])
def test_gemm_codes_tiles_that_cannot_saturate(RA, RB, D):
    """Tiles of 32 with 8-bit accumulators: the matrix-core kernel skips the clamp of a tile whose
    sums provably stay in range (small codes), clamps the others, and gives the test up where
    nothing passes.  Small codes everywhere; small codes with rows, columns and stretches of the
    contraction that fill the range (waves, tiles and pairs of tiles of both kinds side by
    side); and the two mixed the other way round."""
    rng = np.random.default_rng(RA + 3 * RB + D)
    check_gemm_codes_given(gaussian_codes(rng, RA, D, 0.9), gaussian_codes(rng, RB, D, 1.6), 32, 8)
    cA, cB = gaussian_codes(rng, RA, D, 0.8), gaussian_codes(rng, RB, D, 1.2)
    big = random_codes(rng, RA, D, 4, extreme=0.7)
    cA[5::67] = big[5::67]                                   # single rows of A
    cA[:, 96:160] = big[:, 96:160]                           # two tiles of every row, in two pairs
    cA[RA // 2:, 416:448] = big[RA // 2:, 416:448]           # one tile of a pair, half the rows
    cB[3::41] = random_codes(rng, RB, D, 4, extreme=0.7)[3::41]
    check_gemm_codes_given(cA, cB, 32, 8)
    # range-filling first stage (the workgroup stops testing), small codes behind it
    cA, cB = gaussian_codes(rng, RA, D, 0.8), gaussian_codes(rng, RB, D, 1.2)
    cA[:, :128] = random_codes(rng, RA, 128, 4, extreme=0.7)
    cB[:, :128] = random_codes(rng, RB, 128, 4, extreme=0.7)
    check_gemm_codes_given(cA, cB, 32, 8)
    # small codes first, range-filling ones from the second stage on
    cA, cB = gaussian_codes(rng, RA, D, 0.8), gaussian_codes(rng, RB, D, 1.2)
    cA[:, 128:] = random_codes(rng, RA, D - 128, 4, extreme=0.7)
    cB[:, 128:] = random_codes(rng, RB, D - 128, 4, extreme=0.7)
    check_gemm_codes_given(cA, cB, 32, 8)


@pytest.mark.parametrize("a", [9, 10, 12])
@pytest.mark.parametrize("RA,RB,D", [(384, 256, 1152), (256, 128, 16384)])
def test_gemm_codes_tiles_that_cannot_saturate_wider_accumulators(RA, RB, D, a):
    """The same test of the tiles in front of the int16-saturation kernel (accumulators of 9 to
    12 bits): quantizer-like codes (everything passes), codes at the range ends everywhere
    (sums of up to 2048: nothing passes, the workgroups give up), and stretches of the one
    inside the other."""
    rng = np.random.default_rng(RA + 3 * RB + D + a)
    check_gemm_codes_given(gaussian_codes(rng, RA, D, 1.5), gaussian_codes(rng, RB, D, 1.8), 32, a)
    ends = lambda lines, cols: random_codes(rng, lines, cols, 4, extreme=1.0)
    check_gemm_codes_given(ends(RA, D), ends(RB, D), 32, a)
    cA, cB = gaussian_codes(rng, RA, D, 1.5), gaussian_codes(rng, RB, D, 1.8)
    cA[:, 256:448], cB[:, 256:448] = ends(RA, 192), ends(RB, 192)
    cA[7::50, 640:] = ends(len(cA[7::50]), D - 640)
    cB[::2, 640:704] = np.sign(cB[::2, 640:704] + 0.5).astype(np.int8) * 7
    check_gemm_codes_given(cA, cB, 32, a)
    cA, cB = ends(RA, D), ends(RB, D)
    cA[:, 128:] = gaussian_codes(rng, RA, D - 128, 1.5)
    cB[:, 128:] = gaussian_codes(rng, RB, D - 128, 1.8)
    check_gemm_codes_given(cA, cB, 32, a)


def patchwork_codes(rng, lines, D):
    """4-bit codes in patches (up to 96 rows by up to 256 positions), each patch with a
    distribution of its own: small, quantizer-like, uniform over the range, range ends only, zeros."""
    out = np.empty((lines, D), np.int8)
    r = 0
    while r < lines:
        h, k = int(rng.integers(1, 97)), 0
        while k < D:
            w = int(rng.integers(1, 9)) * 32
            shape = (min(h, lines - r), min(w, D - k))
            kind = int(rng.integers(0, 5))
            if kind == 0:
                blk = np.clip(np.rint(rng.normal(0, 0.7, shape)), -8, 7)
            elif kind == 1:
                blk = np.clip(np.rint(rng.normal(0, 1.5, shape)), -8, 7)
            elif kind == 2:
                blk = rng.integers(-8, 8, shape)
            elif kind == 3:
                blk = np.where(rng.random(shape) < 0.5, -8, 7)
            else:
                blk = np.zeros(shape)
            out[r:r + shape[0], k:k + shape[1]] = blk
            k += w
        r += h
    return out


@pytest.mark.parametrize("seed", range(12))
def test_gemm_codes_tile_test_on_patchworks(seed):
    """Random shapes (every third with a split contraction) and patchwork codes, so that tiles
    that pass the matmul's saturation test and tiles that fail it meet in every arrangement;
    accumulators of 8, 9, 10 and 12 bits."""
    rng = np.random.default_rng(1000 + seed)
    RA, RB, D = int(rng.integers(1, 600)), int(rng.integers(65, 400)), int(rng.integers(20, 700)) * 8
    if seed % 3 == 0:
        RA, RB, D = int(rng.integers(64, 256)), int(rng.integers(65, 200)), int(rng.integers(1024, 4096)) * 8
    a = [8, 8, 10, 8, 12, 9][seed % 6]
    check_gemm_codes_given(patchwork_codes(rng, RA, D), patchwork_codes(rng, RB, D), 32, a)


def test_gemm_codes_tile_test_streamed_output():
    """Outputs of 128 MB and more take the instances with streaming stores (waves one block
    high and two wide), which go on in the testing stage after giving the test up: patchwork
    codes on a contraction of nine stages, and on the input gradient's single stage."""
    rng = np.random.default_rng(77)
    check_gemm_codes_given(patchwork_codes(rng, 32768, 1152), patchwork_codes(rng, 1024, 1152), 32, 8)
    check_gemm_codes_given(patchwork_codes(rng, 65536, 128), patchwork_codes(rng, 1152, 128), 32, 8)
    check_gemm_codes_given(patchwork_codes(rng, 32768, 1152), patchwork_codes(rng, 1024, 1152), 32, 10)


def test_gemm_codes_tile_test_many_workgroups():
    """An output that stays in the caches, large enough for several rounds of workgroups per
    compute unit (1024 output tiles, 18 stages each)."""
    rng = np.random.default_rng(78)
    check_gemm_codes_given(patchwork_codes(rng, 8192, 2304), patchwork_codes(rng, 2048, 2304), 32, 8)
    check_gemm_codes_given(patchwork_codes(rng, 4096, 2304), patchwork_codes(rng, 2048, 2304), 32, 12)


@pytest.mark.parametrize("tiles", [255, 256])
def test_gemm_codes_every_tile_saturates_upwards(tiles):
    """255 tiles per output element is the most whose upward saturations the kernel that tests
    its tiles can count (one more takes the other kernel); every tile sum is 32 * 49 -> 127, or
    32 * -56 -> -128, or (every fourth pair of tiles) 32 * 1 -> 32 unclamped."""
    RA = RB = 2944                                            # 23 x 23 output tiles: the contraction is not split
    D = 32 * tiles
    one = dev(np.array([1.0], np.float32))
    cA, cB = np.full((RA, D), 7, np.int8), np.full((RB, D), 7, np.int8)
    qA, qB = dev(capi.pack_codes(cA, 4)), dev(capi.pack_codes(cB, 4))
    _, acc = B.gemm_codes(qA, qB, 4, 4, one, one, D, 1, 8, 32)
    assert torch.all(acc == tiles * 127).item()
    cA[:] = -8
    qA = dev(capi.pack_codes(cA, 4))
    _, acc = B.gemm_codes(qA, qB, 4, 4, one, one, D, 1, 8, 32)
    assert torch.all(acc == tiles * -128).item()
    cA[:] = 7
    small = (np.arange(D) // 64) % 4 == 3
    cA[:, small] = 1
    cB[:, small] = 1
    _, acc = B.gemm_codes(dev(capi.pack_codes(cA, 4)), dev(capi.pack_codes(cB, 4)), 4, 4, one, one, D, 1, 8, 32)
    n_small = int(small.sum()) // 32
    assert torch.all(acc == (tiles - n_small) * 127 + n_small * 32).item()


def test_gemm_codes_hand_cases():
    # all (7, 7): each 16-tile sums to 784 -> 127
    D = 64
    cA = np.full((32, D), 7, np.int8)
    cB = np.full((32, D), 7, np.int8)
    one = dev(np.array([1.0], np.float32))
    out, acc = B.gemm_codes(dev(capi.pack_codes(cA, 4)), dev(capi.pack_codes(cB, 4)), 4, 4, one, one,
                            D, 1, 8, 16)
    assert np.all(host(acc) == 4 * 127) and np.all(host(out) == 508.0)
    cA[:] = -8
    out, acc = B.gemm_codes(dev(capi.pack_codes(cA, 4)), dev(capi.pack_codes(cB, 4)), 4, 4, one, one,
                            D, 1, 8, 16)
    assert np.all(host(acc) == -512)


# ------------------------------------------------------------------ whole matmuls

KIND_NAME = {B.GEMM_FWD: "fwd", B.GEMM_BWD_INPUT: "bwd_input", B.GEMM_BWD_WEIGHT: "bwd_weight"}


def operands(kind, layer):
    return {B.GEMM_FWD: (layer.X, layer.W), B.GEMM_BWD_INPUT: (layer.G, layer.W),
            B.GEMM_BWD_WEIGHT: (layer.X, layer.G)}[kind]


def check_whole_gemm(kind, layer, params: B.Params, sample: int = 0):
    M, K, N = layer.M, layer.K, layer.N
    print(f"gemm {KIND_NAME[kind]} {layer.name} n={params.had_block} s={params.s} a={params.acc_bits} "
          f"bA={params.A.b} bB={params.B.b} rA={params.A.round} rB={params.B.round}", flush=True)
    P, Q = operands(kind, layer)
    out, acc, ws = B.gemm(kind, dev(P), dev(Q), M, K, N, params, want_acc=True)
    L = B.workspace_layout(kind, M, K, N, params)
    ws_h = host(ws)
    got_out, got_acc = host(out), host(acc)
    Pn, Qn = P.numpy(), Q.numpy()
    axes = {B.GEMM_FWD: (1, 0), B.GEMM_BWD_INPUT: (1, 1), B.GEMM_BWD_WEIGHT: (0, 0)}[kind]
    op = o_params(params)
    cA, sA, nA = capi.quantize(Pn, axes[0], params.had_block, op.A, params.seed)
    cB, sB, nB = capi.quantize(Qn, axes[1], params.had_block, op.B, params.seed)
    assert nA == nB == L.n_eff
    # codes and scales inside the workspace
    pA, pB = capi.pack_codes(cA, params.A.b), capi.pack_codes(cB, params.B.b)
    gA = ws_h[L.codesA:L.codesA + pA.size].reshape(pA.shape)
    gB = ws_h[L.codesB:L.codesB + pB.size].reshape(pB.shape)
    assert np.array_equal(gA, pA), "codes of operand A differ"
    assert np.array_equal(gB, pB), "codes of operand B differ"
    assert ws_h[L.scaleA:L.scaleA + 4].view(np.float32)[0] == sA
    assert ws_h[L.scaleB:L.scaleB + 4].view(np.float32)[0] == sB
    if sample:
        rng = np.random.default_rng(99)
        ii = rng.integers(0, L.RA, size=sample)
        jj = rng.integers(0, L.RB, size=sample)
        want_acc = capi.tiled_matmul_sampled(cA, cB, params.s, params.acc_bits, ii, jj)
        assert np.array_equal(got_acc[ii, jj], want_acc)
        assert_close_f32(got_out[ii, jj], capi.dequantize(want_acc, sA, sB, nA))
    else:
        want_acc = capi.tiled_matmul(cA, cB, params.s, params.acc_bits)
        assert np.array_equal(got_acc, want_acc), f"{(got_acc != want_acc).sum()} accumulators differ"
        assert_close_f32(got_out, capi.dequantize(want_acc, sA, sB, nA))


def step_params(kind, n, s, a=8, b=4, layer_id=0, sr_x=False, clip_fwd=1.0, seed=0):
    """Measured configuration: G stochastic in both backward matmuls, the rest nearest."""
    tid = lambda role: 16 * layer_id + {"X": 0, "W": 1, "G": 2}[role] + 4 * kind
    NE, ST = B.ROUND_NEAREST, B.ROUND_STOCHASTIC
    if kind == B.GEMM_FWD:
        A, Bq = B.Operand(b, NE, clip_fwd, tid("X")), B.Operand(b, NE, clip_fwd, tid("W"))
    elif kind == B.GEMM_BWD_INPUT:
        A, Bq = B.Operand(b, ST, 1.0, tid("G")), B.Operand(b, NE, 1.0, tid("W"))
    else:
        A, Bq = B.Operand(b, ST if sr_x else NE, 1.0, tid("X")), B.Operand(b, ST, 1.0, tid("G"))
    return B.Params(had_block=n, acc_bits=a, s=s, seed=seed, A=A, B=Bq)


@pytest.mark.parametrize("kind", [B.GEMM_FWD, B.GEMM_BWD_INPUT, B.GEMM_BWD_WEIGHT])
def test_fc_layer_step(kind):
    layer = workloads.fc_layer(64, 256, 128, seed=0)
    check_whole_gemm(kind, layer, step_params(kind, 16, 16))
    # the paper's own settings: forward without transform, clip 0.975, tile 32;
    # activations stochastic too in the weight-gradient matmul
    if kind == B.GEMM_FWD:
        check_whole_gemm(kind, layer, step_params(kind, 1, 32, clip_fwd=0.975))
    else:
        check_whole_gemm(kind, layer, step_params(kind, 64, 32, sr_x=True))
        check_whole_gemm(kind, layer, step_params(kind, 64, 10 ** 6, a=12, sr_x=True))


@pytest.mark.parametrize("b,a", [(8, 16), (5, 12), (6, 12), (3, 8)])
@pytest.mark.parametrize("kind", [B.GEMM_FWD, B.GEMM_BWD_INPUT, B.GEMM_BWD_WEIGHT])
def test_fc_layer_step_other_input_widths(kind, b, a):
    # input widths and accumulators of the paper's Fig. 4 ranges
    layer = workloads.fc_layer(128, 256, 128, seed=1)
    check_whole_gemm(kind, layer, step_params(kind, 64, 32, a=a, b=b))
    check_whole_gemm(kind, layer, step_params(kind, 64, 128, a=a, b=b, sr_x=True))


@pytest.mark.parametrize("kind", [B.GEMM_FWD, B.GEMM_BWD_INPUT, B.GEMM_BWD_WEIGHT])
def test_har_conv_layer_step(kind):
    layer = workloads.har_conv_layer(seed=0)
    check_whole_gemm(kind, layer, step_params(kind, 32, 32))


@pytest.mark.parametrize("kind", [B.GEMM_FWD, B.GEMM_BWD_INPUT, B.GEMM_BWD_WEIGHT])
def test_ragged_layers(kind):
    # stem-like K = 27 (odd, no transform), classifier-like N = 100 (block order 4)
    layer = workloads.fc_layer(256, 27, 64, seed=3)
    check_whole_gemm(kind, layer, step_params(kind, 64, 32))
    layer = workloads.fc_layer(128, 512, 100, seed=4)
    check_whole_gemm(kind, layer, step_params(kind, 64, 32))
    layer = workloads.fc_layer(128, 561, 11, seed=5)      # HAR FCN widths of the paper's energy table
    check_whole_gemm(kind, layer, step_params(kind, 32, 32))


# ------------------------------------------------------------------ both axes from one read

def check_quantize_dual(T: np.ndarray, n: int, op1: B.Operand, op0: B.Operand, seed: int = 0):
    print(f"quantize_dual shape={T.shape} n={n} b=({op1.b},{op0.b}) round=({op1.round},{op0.round})",
          flush=True)
    c1, s1, c0, s0 = B.quantize_dual(dev(T), n, op1, op0, seed)
    for axis, op, cg, sg in ((1, op1, c1, s1), (0, op0, c0, s0)):
        codes_o, scale_o, _ = capi.quantize(T, axis, n, o_operand(op), seed)
        want = capi.pack_codes(codes_o, op.b)
        got = host(cg)
        assert host(sg)[0] == scale_o, (axis, host(sg)[0], scale_o)
        if not np.array_equal(got, want):
            bad = np.argwhere(got != want)
            raise AssertionError(f"axis {axis}: {len(bad)} code bytes differ, first at {bad[0]}")


@pytest.mark.parametrize("rows,cols,n", [(64, 64, 64), (128, 192, 64), (256, 64, 16), (64, 256, 32),
                                         (320, 128, 64), (512, 1152, 64), (1024, 128, 64), (192, 64, 1),
                                         (100, 64, 64), (64, 72, 64), (256, 256, 256), (37, 27, 64)])
def test_quantize_dual(rows, cols, n):
    rng = np.random.default_rng(rows * 31 + cols)
    T = (rng.standard_normal((rows, cols)) * 0.37).astype(np.float32)
    NE, ST = B.ROUND_NEAREST, B.ROUND_STOCHASTIC
    check_quantize_dual(T, n, B.Operand(4, NE, 1.0, 1), B.Operand(4, NE, 1.0, 2))
    check_quantize_dual(T, n, B.Operand(4, ST, 1.0, 3), B.Operand(4, ST, 1.0, 4), seed=77)
    check_quantize_dual(T, n, B.Operand(4, NE, 0.975, 5), B.Operand(3, ST, 1.0, 6), seed=5)
    check_quantize_dual(T, n, B.Operand(2, ST, 1.0, 7), B.Operand(4, NE, 1.0, 8), seed=6)


@pytest.mark.parametrize("rows,cols,n", [(64, 64, 64), (128, 192, 64), (256, 64, 16), (512, 1152, 64),
                                         (192, 64, 1), (64, 256, 32)])
def test_quantize_dual_byte_codes(rows, cols, n):
    """Both axes with 5 to 8 bits: the two-axis kernels' instances that write a byte per code."""
    rng = np.random.default_rng(rows * 17 + cols)
    T = (rng.standard_normal((rows, cols)) * 2.1).astype(np.float32)
    NE, ST = B.ROUND_NEAREST, B.ROUND_STOCHASTIC
    check_quantize_dual(T, n, B.Operand(8, NE, 1.0, 1), B.Operand(8, NE, 1.0, 2))
    check_quantize_dual(T, n, B.Operand(8, ST, 1.0, 3), B.Operand(8, ST, 1.0, 4), seed=78)
    check_quantize_dual(T, n, B.Operand(5, NE, 0.975, 5), B.Operand(8, ST, 1.0, 6), seed=5)
    check_quantize_dual(T, n, B.Operand(6, ST, 1.0, 7), B.Operand(7, NE, 1.0, 8), seed=6)


def test_quantize_dual_wider_codes_and_zero():
    rng = np.random.default_rng(2)
    T = rng.standard_normal((128, 128)).astype(np.float32)
    check_quantize_dual(T, 64, B.Operand(8), B.Operand(4))
    check_quantize_dual(T, 64, B.Operand(4), B.Operand(6, B.ROUND_STOCHASTIC, 1.0, 9), seed=3)
    check_quantize_dual(np.zeros((64, 128), np.float32), 64, B.Operand(4), B.Operand(4, B.ROUND_STOCHASTIC))


# ------------------------------------------------------------------ second reading of the accumulator

def check_requant_codes(RA, RB, D, bA, bB, s, a, n=1, seed=0, extreme=0.0):
    print(f"requant RA={RA} RB={RB} D={D} bA={bA} bB={bB} s={s} a={a}", flush=True)
    rng = np.random.default_rng(seed + RA * 3 + RB * 5 + D)
    cA = random_codes(rng, RA, D, bA, extreme)
    cB = random_codes(rng, RB, D, bB, extreme)
    sA, sB = np.float32(0.0123), np.float32(3.21e-4)
    want_acc, _ = capi.tiled_matmul_requant(cA, cB, s, a)
    want_out = capi.dequantize_requant(want_acc, sA, sB, n, a)
    out, acc = B.gemm_codes_requant(dev(capi.pack_codes(cA, bA)), dev(capi.pack_codes(cB, bB)), bA, bB,
                                    dev(np.array([sA])), dev(np.array([sB])), D, n, a, s)
    got_acc, got_out = host(acc), host(out)
    assert np.array_equal(got_acc.astype(np.int64), want_acc), \
        f"{(got_acc != want_acc).sum()} of {want_acc.size} totals differ"
    assert_close_f32(got_out, want_out)


@pytest.mark.parametrize("s", [16, 32, 64, 256])
@pytest.mark.parametrize("a", [4, 8, 12])
def test_requant_codes_aligned(s, a):
    check_requant_codes(200, 136, 512, 4, 4, s, a, n=64)
    check_requant_codes(200, 136, 512, 4, 4, s, a, n=64, extreme=0.5)


@pytest.mark.parametrize("s", [1, 5, 27, 48, 100, 1000])
def test_requant_codes_ragged(s):
    check_requant_codes(37, 29, 100, 4, 4, s, 8, n=4)
    check_requant_codes(130, 5, 27, 4, 4, s, 8)
    check_requant_codes(9, 300, 144, 3, 5, s, 6, n=16, extreme=0.3)


def test_requant_codes_wide_inputs_and_many_tiles():
    check_requant_codes(96, 72, 512, 8, 8, 32, 8, n=64, extreme=0.2)
    check_requant_codes(96, 72, 512, 6, 5, 64, 12, n=64, extreme=0.2)
    check_requant_codes(64, 64, 8192, 4, 4, 32, 8, n=64)            # 256 tiles
    check_requant_codes(16, 16, 4096, 4, 4, 1, 8)                   # 4096 tiles of one code: tables in chunks
    zeros = np.zeros((32, 64), np.int8)
    out, acc = B.gemm_codes_requant(dev(capi.pack_codes(zeros, 4)), dev(capi.pack_codes(zeros, 4)), 4, 4,
                                    dev(np.ones(1, np.float32)), dev(np.ones(1, np.float32)), 64, 64, 8, 32)
    assert not host(acc).any() and not host(out).any()


@pytest.mark.parametrize("RA,RB,D,s,a", [
    (300, 200, 1152, 256, 14),      # a short last tile (1152 = 4 * 256 + 128), ragged edge tiles
    (300, 200, 960, 96, 8),         # tiles of three steps that straddle the 128-code stages
    (130, 260, 4128, 32, 8),        # 129 tiles, several column tiles per workgroup
    (256, 128, 16384, 32, 8),       # a long contraction under a small output: split, slices, reduce
    (256, 128, 16384, 128, 11),
    (1152, 128, 65536, 32, 8),      # the weight gradient's shape on the benchmark layer
    (64, 40, 64, 32, 2),            # the narrowest accumulator, two tiles
    (200, 136, 512, 32, 16),
    (200, 136, 512, 64, 3),
    (64, 64, 32768, 32, 8),         # 1024 tiles in one part: beyond the table, the emulation runs
])
def test_requant_codes_two_pass(RA, RB, D, s, a):
    """Shapes the matrix-core kernel takes in two passes (packed 4-bit codes, tiles of whole
    32-code steps, accumulators up to 16 bits), every total against the oracle; the workspace
    is the exact one, which holds no tile sums."""
    lib = B.load()
    exact = lib.hdqt_gemm_codes_requant_workspace_size_for(RA, RB, D, s, 4, 4, a)
    bound = lib.hdqt_gemm_codes_requant_workspace_size(RA, RB, D, s)
    assert 0 < exact <= bound
    if D // s <= 512:
        assert exact < bound / 2 or D // s <= 2, (exact, bound)
    check_requant_codes(RA, RB, D, 4, 4, s, a, n=32, extreme=0.1)


def test_requant_codes_two_pass_streamed_output():
    """The input gradient's shape on the benchmark layer: an output large enough to be written
    with streaming stores (waves one block high and two wide), one stage per output tile."""
    check_requant_codes(65536, 1152, 128, 4, 4, 32, 8, n=64)
    check_requant_codes(65536, 1152, 128, 4, 4, 64, 6, n=64, extreme=0.05)


@pytest.mark.parametrize("kind", [B.GEMM_FWD, B.GEMM_BWD_INPUT, B.GEMM_BWD_WEIGHT])
def test_requant_matmul_from_tensors(kind):
    """The paper's forward setting (tiles of 32, 8-bit accumulators) under the second reading,
    and the two backward matmuls, from the fp32 tensors: quantization as everywhere else, then
    the oracle's second-reading matmul on the oracle's codes."""
    layer = workloads.fc_layer(320, 256, 192, seed=2)
    M, K, N = layer.M, layer.K, layer.N
    P, Q = {B.GEMM_FWD: (layer.X, layer.W), B.GEMM_BWD_INPUT: (layer.G, layer.W),
            B.GEMM_BWD_WEIGHT: (layer.X, layer.G)}[kind]
    axes = {B.GEMM_FWD: (1, 0), B.GEMM_BWD_INPUT: (1, 1), B.GEMM_BWD_WEIGHT: (0, 0)}[kind]
    prm = B.Params(had_block=64, acc_bits=8, s=32, seed=4, A=B.Operand(4, B.ROUND_NEAREST, 0.975, 1),
                   B=B.Operand(4, B.ROUND_STOCHASTIC, 1.0, 2))
    out, acc, _ = B.gemm_requant(kind, dev(P), dev(Q), M, K, N, prm, want_acc=True)
    cA, sA, nA = capi.quantize(P.numpy(), axes[0], 64, o_operand(prm.A), 4)
    cB, sB, nB = capi.quantize(Q.numpy(), axes[1], 64, o_operand(prm.B), 4)
    want_acc, _ = capi.tiled_matmul_requant(cA, cB, 32, 8)
    assert np.array_equal(host(acc).astype(np.int64), want_acc)
    assert_close_f32(host(out), capi.dequantize_requant(want_acc, sA, sB, nA, 8))
