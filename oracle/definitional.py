"""Second, even plainer statement of the HDQT matmul in NumPy / Python loops.

TEST INFRASTRUCTURE ONLY.  Written independently of oracle/hdqt_oracle.c (other
formulas where the paper allows: closed-form Hadamard entries instead of the
recursion, level-by-level pair sums instead of a recursive tree, Python
integers for Philox) so that the two can be played against each other by brute
force on tiny shapes.  Far too slow for anything else.

Follows the paper's Methodology section: Q(x) with max calibration, Sylvester
Hadamard in block-diagonal form along the contraction dimension, stochastic
rounding, tiles of size s with low-bit accumulators.
"""
import numpy as np

F = np.float32


def hadamard_entry(i: int, j: int) -> int:
    """Entry of the Sylvester matrix: (-1)^(number of common set bits)."""
    return -1 if bin(i & j).count("1") % 2 else 1


def hadamard(n: int) -> np.ndarray:
    return np.array([[hadamard_entry(i, j) for j in range(n)] for i in range(n)], dtype=np.int64)


def n_eff(D: int, n: int) -> int:
    m = n
    while D % m:
        m //= 2
    return m


def _pair_sum_f32(terms: np.ndarray) -> np.float32:
    """Balanced tree over a power-of-two number of binary32 terms."""
    t = terms.astype(F)
    while t.shape[0] > 1:
        t = (t[0::2] + t[1::2]).astype(F)
    return t[0]


def transform_line(x: np.ndarray, n: int) -> np.ndarray:
    """x: 1-D binary32 line of length D (n | D) -> x H, H block-diagonal."""
    D = x.shape[0]
    y = np.empty(D, dtype=F)
    Hn = hadamard(n)
    for blk in range(D // n):
        seg = x[blk * n:(blk + 1) * n].astype(F)
        for i in range(n):
            y[blk * n + i] = _pair_sum_f32(np.where(Hn[i] > 0, seg, -seg))
    return y


def philox4x32_10(ctr, key):
    c = [int(v) & 0xFFFFFFFF for v in ctr]
    k = [int(v) & 0xFFFFFFFF for v in key]
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def sr_bits(seed: int, tensor_id: int, e: int) -> int:
    blk = e // 8
    out = philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, tensor_id, 0],
                        [seed & 0xFFFFFFFF, seed >> 32])
    return (out[(e // 2) % 4] >> (16 * (e % 2))) & 0xFFFF


def quantize(T: np.ndarray, axis: int, had_block: int, b: int, stochastic: bool = False,
             clip: float = 1.0, tensor_id: int = 0, seed: int = 0):
    """-> (codes int64 [lines, D] contraction-major, scale, n_eff)."""
    T = np.asarray(T, dtype=F)
    rows, cols = T.shape
    lines_first = T if axis == 1 else T.T          # [lines, D] view of the source
    D = lines_first.shape[1]
    n = n_eff(D, had_block)
    Y = np.stack([transform_line(np.ascontiguousarray(line), n) for line in lines_first])
    amax = F(np.max(np.abs(Y)))
    amax_c = F(F(clip) * amax)
    codes = np.zeros(Y.shape, dtype=np.int64)
    if amax_c == 0:
        return codes, F(0), n
    levels = F(2 ** (b - 1))
    inv = F(levels / amax_c)
    scale = F(amax_c / levels)
    for l in range(Y.shape[0]):
        for d in range(D):
            v = F(Y[l, d] * inv)
            if stochastic:
                r, c = (l, d) if axis == 1 else (d, l)
                e = r * cols + c
                fl = np.floor(v)
                frac = F(v - fl)
                q = int(fl) + (1 if F(sr_bits(seed, tensor_id, e)) < F(frac * F(65536.0)) else 0)
            else:
                q = int(np.rint(v))
            codes[l, d] = min(max(q, -(2 ** (b - 1))), 2 ** (b - 1) - 1)
    return codes, scale, n


def tiled_matmul(qA: np.ndarray, qB: np.ndarray, s: int, a: int) -> np.ndarray:
    RA, D = qA.shape
    RB = qB.shape[0]
    lo, hi = -(2 ** (a - 1)), 2 ** (a - 1) - 1
    acc = np.zeros((RA, RB), dtype=np.int64)
    for i in range(RA):
        for j in range(RB):
            total = 0
            for t0 in range(0, D, s):
                part = sum(int(qA[i, d]) * int(qB[j, d]) for d in range(t0, min(t0 + s, D)))
                total += min(max(part, lo), hi)
            acc[i, j] = total
    return acc


def dequantize(acc: np.ndarray, scaleA, scaleB, n: int) -> np.ndarray:
    dq = F(F(F(scaleA) * F(scaleB)) * F(1.0 / n))
    return (acc.astype(F) * dq).astype(F)


def tiled_matmul_requant(qA: np.ndarray, qB: np.ndarray, s: int, a: int):
    """Second reading of the low-bit accumulator (Methodology, tiled quantization): every
    tile's partial-sum tensor is quantized to a bits with its own max and the tile results
    are added.  Pure Python over tiles and elements; exact rational arithmetic decides the
    rounding wherever binary32 cannot be trusted to show it.
    -> (acc as Python ints [RA][RB] with value acc / 2^(a-1), [m_t])."""
    from fractions import Fraction
    RA, D = qA.shape
    RB = qB.shape[0]
    qmax, qmin = (1 << (a - 1)) - 1, -(1 << (a - 1))
    acc = [[0] * RB for _ in range(RA)]
    maxima = []
    for t0 in range(0, D, s):
        t1 = min(t0 + s, D)
        P = [[sum(int(qA[i, d]) * int(qB[j, d]) for d in range(t0, t1)) for j in range(RB)] for i in range(RA)]
        m = max(abs(v) for row in P for v in row)
        maxima.append(m)
        if m == 0:
            continue
        inv = np.float32(np.float64(1 << (a - 1)) / np.float64(m))      # one correctly rounded division
        for i in range(RA):
            for j in range(RB):
                v = np.float32(np.float32(P[i][j]) * inv)                # one binary32 multiplication
                # nearest integer, ties to even, decided exactly on the binary32 value v
                f = Fraction(float(v))
                lo = f.numerator // f.denominator
                frac = f - lo
                c = lo if frac < Fraction(1, 2) else lo + 1 if frac > Fraction(1, 2) else lo + (lo & 1)
                c = max(qmin, min(qmax, c))
                acc[i][j] += c * m
    return acc, maxima
