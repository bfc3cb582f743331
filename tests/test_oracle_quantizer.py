"""Pins for the oracle's quantizer Q, max calibration and stochastic rounding
(paper, Methodology section; forward clip factor 0.975 from Experiments)."""
import os
import subprocess
import sys

import numpy as np
import pytest

from oracle import capi, definitional

NEAREST = capi.ROUND_NEAREST
STOCH = capi.ROUND_STOCHASTIC


def _grid_cases(golden_dir):
    cases = []
    with open(os.path.join(golden_dir, "quantizer_grid.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            b, step, js, cs = [f.strip() for f in line.split(";")]
            cases.append((int(b), float(step), [float(v) for v in js.split(",")],
                          [int(v) for v in cs.split(",")]))
    return cases


def test_grid_inputs_give_known_codes(golden_dir):
    cases = _grid_cases(golden_dir)
    assert len(cases) >= 5
    for b, step, js, want in cases:
        x = (np.array(js, dtype=np.float64) * step).astype(np.float32)
        for axis, T in ((1, x[None, :]), (0, x[:, None])):
            codes, scale, ne = capi.quantize(T, axis, 1, capi.Operand(b=b))
            assert ne == 1
            assert codes.reshape(-1).tolist() == want, (b, step)
            assert scale == np.float32(step)        # one code step
        c2, s2, _ = definitional.quantize(x[None, :], 1, 1, b)
        assert c2.reshape(-1).tolist() == want and s2 == np.float32(step)


@pytest.mark.parametrize("b", [2, 3, 4, 5, 6, 8])
def test_code_range_monotone_antisymmetric(b):
    rng = np.random.default_rng(b)
    x = np.sort(rng.standard_normal(4001).astype(np.float32))
    codes, scale, _ = capi.quantize(x[None, :], 1, 1, capi.Operand(b=b))
    c = codes[0].astype(np.int64)
    assert c.min() >= -(2 ** (b - 1)) and c.max() <= 2 ** (b - 1) - 1   # 2^b levels, never +2^(b-1)
    assert np.all(np.diff(c) >= 0)                                      # monotone
    # sign antisymmetry away from the clamp: Q(-x) = -Q(x)
    xs = np.concatenate([x, -x])
    cs, _, _ = capi.quantize(xs[None, :], 1, 1, capi.Operand(b=b))
    pos, neg = cs[0, :x.size].astype(np.int64), cs[0, x.size:].astype(np.int64)
    inside = (np.abs(pos) < 2 ** (b - 1) - 1) & (np.abs(neg) < 2 ** (b - 1) - 1)
    assert np.array_equal(pos[inside], -neg[inside])


def test_textbook_absmax_quantization_when_no_transform():
    # n = 1, clip = 1 reduces to symmetric absmax integer quantization:
    # code = clamp(rint(x / max|x| * 2^(b-1))), dequantized error <= scale/2
    rng = np.random.default_rng(42)
    x = rng.standard_normal((7, 33)).astype(np.float32)
    for b in (4, 8):
        codes, scale, _ = capi.quantize(x, 1, 1, capi.Operand(b=b))
        amax = np.abs(x).max()
        ref = np.clip(np.rint(x.astype(np.float64) / amax * 2 ** (b - 1)), -(2 ** (b - 1)),
                      2 ** (b - 1) - 1)
        # fp64 evaluation may differ from the fp32 path only at near-ties
        assert np.mean(codes != ref) < 1e-2
        assert np.max(np.abs(codes.astype(np.int64) - ref)) <= 1
        err = np.abs(codes.astype(np.float64) * scale - x)
        inside = codes < 2 ** (b - 1) - 1
        assert np.all(err[inside] <= scale / 2 * (1 + 1e-6))
        assert np.isclose(scale, amax / 2 ** (b - 1), rtol=1e-7)


def test_paper_formula_dequantized_values():
    # Q(x) = round(clip(alpha x) 2^(b-1)) 2^-(b-1) / alpha, evaluated in fp64,
    # against codes*scale; they may differ only by the +2^(b-1) level and at ties
    rng = np.random.default_rng(9)
    x = rng.standard_normal(5000).astype(np.float32)
    b = 4
    codes, scale, _ = capi.quantize(x[None, :], 1, 1, capi.Operand(b=b))
    alpha = 1.0 / np.abs(x.astype(np.float64)).max()
    q = np.rint(np.clip(alpha * x.astype(np.float64), -1, 1) * 2 ** (b - 1)) * 2.0 ** -(b - 1) / alpha
    mine = codes[0].astype(np.float64) * float(scale)
    top = np.isclose(q, 1.0 / alpha)
    assert np.mean(~np.isclose(mine[~top], q[~top], rtol=1e-6, atol=1e-12)) < 2e-3
    assert np.all(codes[0][top] == 2 ** (b - 1) - 1)


def test_zero_tensor():
    for rm in (NEAREST, STOCH):
        codes, scale, _ = capi.quantize(np.zeros((4, 16), np.float32), 1, 16,
                                        capi.Operand(b=4, round_mode=rm))
        assert not codes.any() and scale == 0.0


def test_clip_factor_saturates_outliers():
    # forward-pass clip 0.975: scale = fl(0.975*amax)/2^(b-1); values above clip*amax clamp
    x = np.array([[1.0, -1.0, 0.98, 0.5, -0.97, 0.0, 0.25, -0.3]], dtype=np.float32)
    codes, scale, _ = capi.quantize(x, 1, 1, capi.Operand(b=4, clip=0.975))
    assert scale == np.float32(np.float32(0.975) * np.float32(1.0)) / np.float32(8)
    assert codes[0, 0] == 7 and codes[0, 1] == -8 and codes[0, 2] == 7
    assert codes[0, 3] == 4                       # 0.5/0.975*8 = 4.10 -> 4
    assert codes[0, 4] == -8                      # -0.97/0.975*8 = -7.96 -> -8
    assert codes[0, 6] == 2 and codes[0, 7] == -2


def test_hadamard_domain_axis_and_layout():
    # codes are contraction-major: quantizing T along axis 0 equals quantizing
    # T^T along axis 1 (nearest rounding does not look at element indices)
    rng = np.random.default_rng(1)
    T = rng.standard_normal((32, 6)).astype(np.float32)
    c0, s0, n0 = capi.quantize(T, 0, 16, capi.Operand(b=4))
    c1, s1, n1 = capi.quantize(np.ascontiguousarray(T.T), 1, 16, capi.Operand(b=4))
    assert c0.shape == (6, 32) and np.array_equal(c0, c1) and s0 == s1 and n0 == n1 == 16


def test_hadamard_domain_codes_from_known_transform():
    # block [8,0,...,0] transforms to all 8s; [1,1,..,1] transforms to [n,0,..]:
    # the tensor maximum is 16, so the codes are 4 (for 8) and 7 (for 16 -> +8 -> clamp)
    n = 16
    T = np.zeros((2, n), dtype=np.float32)
    T[0, 0] = 8.0
    T[1, :] = 1.0
    codes, scale, ne = capi.quantize(T, 1, n, capi.Operand(b=4))
    assert ne == n and scale == np.float32(2.0)
    assert np.all(codes[0] == 4)
    assert codes[1, 0] == 7 and not codes[1, 1:].any()


# ---------------------------------------------------------------- stochastic

def test_stochastic_never_moves_integers_and_stays_adjacent():
    rng = np.random.default_rng(2)
    x = rng.uniform(-8, 8, size=(64, 64)).astype(np.float32)
    x[0, 0] = 8.0                                  # amax = 8 -> inv = 1, v = x
    x[1, :] = np.arange(-32, 32) // 4              # exact integers in [-8, 7]
    op = capi.Operand(b=4, round_mode=STOCH, tensor_id=3)
    codes, scale, _ = capi.quantize(x, 1, 1, op, seed=5)
    assert scale == 1.0
    assert np.array_equal(codes[1], x[1].astype(np.int8))
    lo = np.clip(np.floor(x), -8, 7)
    hi = np.clip(np.ceil(x), -8, 7)
    assert np.all((codes == lo) | (codes == hi))
    # deterministic in (seed, tensor_id, element), different when any differs
    again, _, _ = capi.quantize(x, 1, 1, op, seed=5)
    assert np.array_equal(codes, again)
    other_seed, _, _ = capi.quantize(x, 1, 1, op, seed=6)
    other_id, _, _ = capi.quantize(x, 1, 1, capi.Operand(b=4, round_mode=STOCH, tensor_id=4), seed=5)
    assert not np.array_equal(codes, other_seed) and not np.array_equal(codes, other_id)


def test_stochastic_element_index_is_position_in_source_tensor():
    # the random bits belong to the source element, whatever axis is contracted:
    # with n = 1 the two axes give transposed codes
    rng = np.random.default_rng(8)
    x = rng.uniform(-8, 8, size=(24, 40)).astype(np.float32)
    x[0, 0] = 8.0
    op = capi.Operand(b=4, round_mode=STOCH, tensor_id=9)
    c1, _, _ = capi.quantize(x, 1, 1, op, seed=1)
    c0, _, _ = capi.quantize(x, 0, 1, op, seed=1)
    assert np.array_equal(c0, c1.T)


def test_stochastic_rounding_is_unbiased():
    # P(up) = ceil(frac * 2^16) / 2^16: the mean over many elements sits within
    # 4 sigma of the value
    n = 1 << 17
    for frac in (0.1, 0.5, 0.9, 0.003):
        x = np.full((1, n), 2.0 + frac, dtype=np.float32)
        x[0, 0] = 8.0
        codes, scale, _ = capi.quantize(x, 1, 1, capi.Operand(b=4, round_mode=STOCH, tensor_id=1),
                                        seed=123)
        up = (codes[0, 1:] == 3).mean()
        f32 = float(np.float32(2.0 + frac)) - 2.0
        sigma = np.sqrt(f32 * (1 - f32) / (n - 1))
        assert abs(up - f32) < 4 * sigma + 2.0 ** -16
    # exact probability from the 16-bit threshold rule
    thr = np.float32(np.float32(0.3) * np.float32(65536.0))
    ups = sum(np.float32(u) < thr for u in range(65536))
    assert ups == int(np.ceil(float(thr)))


def test_sr_bits_layout_and_uniformity():
    # eight consecutive elements share one Philox block: half-word (e mod 2) of
    # output word ((e/2) mod 4); counter = (e/8 low, e/8 high, tensor_id, 0)
    seed, tid = 0x1234567890ABCDEF, 77
    for base in (0, 8, 8 * 12345, 8 * (1 << 33)):
        blk = base >> 3
        out = capi.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, tid, 0],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        for j in range(8):
            want = (int(out[j // 2]) >> (16 * (j % 2))) & 0xFFFF
            assert capi.sr_bits(seed, tid, base + j) == want
            assert definitional.sr_bits(seed, tid, base + j) == want
    bits = np.array([capi.sr_bits(1, 2, e) for e in range(1 << 15)])
    hist = np.bincount(bits >> 12, minlength=16)
    expected = bits.size / 16
    chi2 = ((hist - expected) ** 2 / expected).sum()
    assert chi2 < 50          # 15 degrees of freedom; p ~ 1e-5 at 50


def test_philox_two_implementations_agree():
    rng = np.random.default_rng(0)
    for _ in range(300):
        ctr = rng.integers(0, 2 ** 32, size=4, dtype=np.uint64)
        key = rng.integers(0, 2 ** 32, size=2, dtype=np.uint64)
        assert capi.philox4x32_10(ctr, key).tolist() == definitional.philox4x32_10(ctr, key)


_ATEN_PROBE = r"""
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdio>
#include <cstdlib>
int main(int argc, char** argv) {
  // argv: seed subsequence offset   -> the four words of that 128-bit block
  unsigned long long seed = strtoull(argv[1], 0, 0), sub = strtoull(argv[2], 0, 0),
                     off = strtoull(argv[3], 0, 0);
  at::philox_engine eng(seed, sub, off);
  for (int i = 0; i < 4; ++i) printf("%u\n", eng());
  return 0;
}
"""


def test_philox_against_aten_engine(tmp_path):
    """Independent library pin: PyTorch's host-side Philox4x32-10 engine
    (key = seed words, counter = (offset low, offset high, subsequence low,
    subsequence high)) must give the same block as the oracle."""
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    src = tmp_path / "probe.cpp"
    exe = tmp_path / "probe"
    src.write_text(_ATEN_PROBE)
    r = subprocess.run(["g++", "-O1", "-std=c++17", "-I", inc, str(src), "-o", str(exe)],
                       capture_output=True, text=True)
    if r.returncode != 0:
        pytest.skip("ATen Philox header does not compile stand-alone here: " + r.stderr[-300:])
    cases = [(0, 0, 0), (1, 2, 3), (0xDEADBEEFCAFEF00D, 17, 123456789),
             (42, 0xFFFFFFFF, (1 << 40) + 5), (2 ** 64 - 1, 5, 0)]
    for seed, sub, off in cases:
        got = subprocess.run([str(exe), str(seed), str(sub), str(off)], capture_output=True,
                             text=True, check=True).stdout.split()
        want = capi.philox4x32_10([off & 0xFFFFFFFF, off >> 32, sub & 0xFFFFFFFF, sub >> 32],
                                  [seed & 0xFFFFFFFF, seed >> 32])
        assert [int(v) for v in got] == want.tolist(), (seed, sub, off)


def test_c_oracle_equals_definitional_on_tiny_tensors():
    rng = np.random.default_rng(77)
    for trial in range(12):
        rows, cols = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        rows *= int(rng.choice([1, 2, 4]))
        cols *= int(rng.choice([1, 2, 4, 8]))
        T = (rng.standard_normal((rows, cols)) * 10.0 ** rng.integers(-2, 3)).astype(np.float32)
        for axis in (0, 1):
            for b in (3, 4, 8):
                n = int(rng.choice([1, 2, 8, 64]))
                clip = float(rng.choice([1.0, 0.975]))
                st = bool(rng.integers(0, 2))
                c, s, ne = capi.quantize(T, axis, n, capi.Operand(b=b, round_mode=int(st), clip=clip,
                                                                  tensor_id=trial), seed=trial + 1)
                c2, s2, ne2 = definitional.quantize(T, axis, n, b, stochastic=st, clip=clip,
                                                    tensor_id=trial, seed=trial + 1)
                assert ne == ne2 and s == s2 and np.array_equal(c, c2)


def test_packed_format():
    codes = np.array([[-8, 7, -1, 0, 3], [1, 2, 3, 4, 5]], dtype=np.int8)
    p = capi.pack_codes(codes, 4)
    assert p.shape == (2, 3)
    # low nibble = even index, high nibble = odd index, zero pad nibble
    assert p[0].tolist() == [0x8 | (0x7 << 4), 0xF | (0x0 << 4), 0x3]
    assert p[1].tolist() == [0x1 | (0x2 << 4), 0x3 | (0x4 << 4), 0x5]
    p8 = capi.pack_codes(codes, 8)
    assert p8.shape == (2, 5) and np.array_equal(p8.view(np.int8), codes)


def test_quantize_is_the_transform_followed_by_the_quantizer_at_block_order_one():
    """The oracle's quantizer calls its own transform first: quantizing the transformed tensor
    with block order 1 gives the same codes and the same scale.  (The full-size GPU tests rely
    on this to take the transform of a 2^28-element operand once for several code widths.)"""
    rng = np.random.default_rng(0)
    T = rng.standard_normal((96, 512)).astype(np.float32)
    for axis, n in ((1, 256), (0, 32), (1, 64), (0, 64)):
        D = T.shape[1] if axis == 1 else T.shape[0]
        ne = capi.n_eff(D, n)
        Y = capi.hadamard_transform(T, axis, ne)
        for b, rnd, clip in ((4, 0, 1.0), (8, 0, 0.975), (4, 1, 1.0), (6, 1, 1.0)):
            op = capi.Operand(b, rnd, clip, 3)
            c1, s1, n1 = capi.quantize(T, axis, n, op, 5)
            c2, s2, n2 = capi.quantize(Y, axis, 1, op, 5)
            assert n1 == ne and n2 == 1
            assert s1 == s2 and np.array_equal(c1, c2), (axis, n, b, rnd)
