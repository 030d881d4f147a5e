"""Pins of the oracle's quantizers against exact rational arithmetic, closed
forms and hand-checkable examples (CPU only)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import taq_oracle as O
from oracle import brute


def _fp16_rows(seed, rows, n, scale=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal((rows, n)) * scale).astype(np.float16)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("n", [40, 320])
def test_symq_equals_exact_rational_on_fp16_inputs(bits, n):
    x = _fp16_rows(11 + bits + n, 24, n)
    code, scale = O.symq(x.astype(np.float32), bits)
    qmax = (1 << (bits - 1)) - 1
    for r in range(x.shape[0]):
        ref, amax = brute.symq_exact([float(v) for v in x[r]], bits)
        assert list(code[r]) == ref
        # scale is the float32 nearest to amax/qmax
        exact = amax / qmax
        s = Fraction(float(scale[r]))
        ulp = Fraction(float(np.spacing(scale[r])))
        assert abs(s - exact) <= ulp / 2


def test_symq_ties_are_common_and_go_to_even():
    # x = [-1, .5, .25, 1] at 4 bits: x*7 = [-7, 3.5, 1.75, 7]; 3.5 is a tie -> 4
    code, scale = O.symq(np.array([[-1.0, 0.5, 0.25, 1.0]], dtype=np.float32), 4)
    assert list(code[0]) == [-7, 4, 2, 7]
    assert scale[0] == np.float32(1.0) / np.float32(7.0)
    # 2.5 -> 2 (even), 4.5 -> 4, 5.5 -> 6 : x = k/7 is not fp16-exact, so build ties at 8 bits
    x = np.array([[127.0, 2.5, 4.5, 5.5, -2.5, -5.5]], dtype=np.float32)
    code, _ = O.symq(x, 8)
    assert list(code[0]) == [127, 2, 4, 6, -2, -6]


@pytest.mark.parametrize("bits", [4, 8])
def test_symq_invariants(bits):
    qmax = (1 << (bits - 1)) - 1
    x = _fp16_rows(5, 64, 80, scale=2.5).astype(np.float32)
    code, scale = O.symq(x, bits)
    deq = code.astype(np.float64) * scale.astype(np.float64)[:, None]
    # error bound: half a step (plus float32 rounding of the scale)
    assert np.all(np.abs(x - deq) <= scale[:, None].astype(np.float64) * (0.5 + 1e-6))
    # the row maximum hits the end of the grid
    assert np.all(np.abs(code).max(axis=1) == qmax)
    assert code.min() >= -qmax and code.max() <= qmax
    # sign symmetry
    code_neg, scale_neg = O.symq(-x, bits)
    assert np.array_equal(code_neg, -code) and np.array_equal(scale_neg, scale)
    # idempotence on the dequantised values (computed in float32 as code*scale)
    deq32 = (code.astype(np.float32) * scale[:, None]).astype(np.float32)
    code2, scale2 = O.symq(deq32, bits)
    assert np.array_equal(code2, code)
    assert np.allclose(scale2, scale, rtol=2e-7, atol=0)


def test_symq_zero_row_and_axis():
    x = np.zeros((3, 8), dtype=np.float32)
    x[1, 2] = -3.0
    code, scale = O.symq(x, 8)
    assert np.array_equal(code[0], np.zeros(8, dtype=np.int32)) and scale[0] == 1.0
    assert code[1, 2] == -127 and scale[1] == np.float32(3.0) / np.float32(127.0)
    # axis argument: quantizing columns equals quantizing the transpose's rows
    y = _fp16_rows(3, 6, 10).astype(np.float32)
    c0, s0 = O.symq(y, 8, axis=0)
    c1, s1 = O.symq(y.T.copy(), 8, axis=1)
    assert np.array_equal(c0, c1.T) and np.array_equal(s0, s1)


def test_symq_float32_sequence_matches_scalar_float32_brute_on_full_mantissa_inputs():
    # inputs with full float32 mantissas (as the dequantised projection rows have)
    rng = np.random.Generator(np.random.PCG64(99))
    x = (rng.standard_normal((16, 40)) * 1.7).astype(np.float32)
    for bits in (4, 8):
        code, scale = O.symq(x, bits)
        for r in range(x.shape[0]):
            cr, sc = brute.symq_f32(list(x[r]), bits)
            assert list(code[r]) == cr and scale[r] == sc


def test_uq8_known_values():
    p = np.array([0.0, 1.0, 1.0 / 77.0, 0.5, 2.5 / 255.0, 3.5 / 255.0, 1e-4, 0.999])
    # 0.5*255 = 127.5 -> 128 (even); 2.5/255 and 3.5/255 are not exact, so only the clear cases are pinned
    code = O.uq8(p)
    assert code[0] == 0 and code[1] == 255 and code[2] == 3 and code[3] == 128
    assert code[6] == 0 and code[7] == 255
    # error bound 1/510 on a fine grid, and monotonicity
    grid = np.linspace(0.0, 1.0, 20001)
    c = O.uq8(grid)
    assert np.all(np.abs(c / 255.0 - grid) <= 1.0 / 510.0 + 1e-7)
    assert np.all(np.diff(c) >= 0) and c.min() == 0 and c.max() == 255


def test_pack_int4_layout():
    packed = O.pack_int4(np.array([[-7, 7, 0, -1, 3, -4]]))
    # low nibble = even element, two's complement: -7 -> 0x9, -1 -> 0xF, -4 -> 0xC
    assert list(packed[0]) == [0x79, 0xF0, 0xC3]


def test_quantize_weight_per_output_channel():
    W = _fp16_rows(17, 12, 48, scale=0.05)
    code, scale = O.quantize_weight(W)
    assert code.dtype == np.int8 and code.shape == W.shape and scale.shape == (12,)
    for c in range(12):
        ref, amax = brute.symq_exact([float(v) for v in W[c]], 8)
        assert list(code[c].astype(int)) == ref
    # scaling one output channel changes only that channel's scale, not its codes
    W2 = W.copy()
    W2[3] = (W2[3].astype(np.float32) * 4).astype(np.float16)
    code2, scale2 = O.quantize_weight(W2)
    assert np.array_equal(code2, code)
    assert scale2[3] == pytest.approx(4 * scale[3], rel=1e-6) and np.array_equal(np.delete(scale2, 3), np.delete(scale, 3))


def test_bops_ratios_match_table1():
    # closed form: BOPs scale with b_w*b_a, so 32/32 -> 8/8 is 16x and -> 8/4 is 32x
    args = dict(B=2, N=4096, C=320, T=77, Cc=768)
    full = O.block_bops(**args, b_w=32, b_a=32)
    assert full / O.block_bops(**args, b_w=8, b_a=8) == 16.0
    assert full / O.block_bops(**args, b_w=8, b_a=4) == 32.0
    # the paper's own whole-model figures show the same ratios (to its printed precision)
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table1_bops.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            model, bits, val = line.split()
            rows[(model, bits)] = float(val)
    for model in ("sd15", "sdxl_turbo"):
        assert rows[(model, "32/32")] / rows[(model, "8/8")] == pytest.approx(16.0, rel=0.02)
        assert rows[(model, "32/32")] / rows[(model, "8/4")] == pytest.approx(32.0, rel=0.02)
    # MAC count of the block, by hand, for a 1-token case
    assert O.block_bops(B=1, N=1, C=2, T=3, Cc=5, b_w=1, b_a=1) == 2.0 * (4 + 2 * 3 * 5 * 2 + 2 * 3 * 2 + 4)


def test_uq4_known_values_and_bound():
    # the 4-bit probability grid 1/15: 1/77 rounds to 0, 0.5*15 = 7.5 -> 8 (even), 0.1*15 = 1.5 -> 2 (even)
    p = np.array([0.0, 1.0, 1.0 / 77.0, 0.5, 0.1, 0.0333, 0.0334])
    code = O.uq(p, 4)
    assert list(code) == [0, 15, 0, 8, 2, 0, 1]
    grid = np.linspace(0.0, 1.0, 20001)
    c = O.uq(grid, 4)
    assert np.all(np.abs(c / 15.0 - grid) <= 1.0 / 30.0 + 1e-7) and np.all(np.diff(c) >= 0)
    assert c.min() == 0 and c.max() == 15
    with pytest.raises(ValueError):
        O.uq(p, 5)


@pytest.mark.parametrize("bits", [4, 8])
def test_uq_log2_known_values_bound_and_fixed_points(bits):
    last = (1 << bits) - 1
    # -log2: 1 -> 0, .5 -> 1, .25 -> 2, .3 -> 1.737 -> 2, .36 -> 1.474 -> 1, .7 -> .515 -> 1, .71 -> .494 -> 0
    p = np.array([1.0, 0.5, 0.25, 0.3, 0.36, 0.7, 0.71, 1e-6, 0.0])
    code = O.uq_log2(p, bits)
    assert list(code[:7]) == [0, 1, 2, 2, 1, 1, 0]
    assert code[7] == min(last, 20) and code[8] == last      # -log2(1e-6) = 19.93; zero takes the last code
    # every power of two on the grid is a fixed point
    k = np.arange(0, last + 1)
    assert np.array_equal(O.uq_log2(np.exp2(-k.astype(np.float64)), bits), k)
    # inside the grid's range the dequantised value is within a factor sqrt(2) of p; codes fall as p grows
    grid = np.exp(np.linspace(np.log(2.0 ** -(min(last, 40) + 0.49)), 0.0, 50001))
    c = O.uq_log2(grid, bits)
    ratio = np.exp2(-c.astype(np.float64)) / grid
    assert ratio.max() <= 2 ** 0.5 * (1 + 1e-6) and ratio.min() >= 2 ** -0.5 * (1 - 1e-6)
    assert np.all(np.diff(c) <= 0) and c.max() == min(last, 40) and c.min() == 0
    # decision boundaries sit at the geometric means 2^-(k+1/2) of neighbouring grid points (no logarithm needed
    # to state that): just above one the code is k, just below it k + 1
    kk = np.arange(0, min(last, 60))
    edge = np.sqrt(np.exp2(-kk.astype(np.float64)) * np.exp2(-(kk + 1).astype(np.float64)))
    assert np.array_equal(O.uq_log2(edge * (1 + 1e-5), bits), kk)
    assert np.array_equal(O.uq_log2(edge * (1 - 1e-5), bits), kk + 1)
    with pytest.raises(ValueError):
        O.uq_log2(p, 16)


def test_uq_rowmax_known_values_bound_and_mask():
    # 4 bits, amax = 0.5: 15, 0.25*15/0.5 = 7.5 -> 8 (even), 0.125 -> 3.75 -> 4, 0.05 -> 1.5 -> 2 (even)
    code, scale = O.uq_rowmax(np.array([[0.5, 0.25, 0.125, 0.05, 0.0]]), 4)
    assert list(code[0]) == [15, 8, 4, 2, 0] and scale[0] == np.float32(0.5) / np.float32(15)
    # the largest quantized entry always takes the last code; error at most half a step of the row's own scale
    rng = np.random.Generator(np.random.PCG64(4))
    p = rng.dirichlet(np.ones(77) * 0.3, size=200)
    for bits in (4, 8):
        last = (1 << bits) - 1
        c, sc = O.uq_rowmax(p, bits)
        assert np.all(c.max(axis=1) == last) and c.min() >= 0
        assert np.all(np.abs(c * sc[:, None].astype(np.float64) - p) <= sc[:, None] * (0.5 + 1e-5))
        # never coarser than the fixed 1/(2^b-1) grid, whose step the row scale cannot exceed
        assert np.all(sc <= np.float32(1.0) / np.float32(last) * (1 + 1e-6))
        # scaling a row by a power of two scales its scale and leaves the codes alone
        c2, sc2 = O.uq_rowmax(p * 0.25, bits)
        assert np.array_equal(c2, c) and np.array_equal(sc2, sc * np.float32(0.25))
    # entries outside the mask neither set the range nor get codes
    m = np.ones(77, dtype=bool)
    m[[0, 5]] = False
    big = p.copy()
    big[:, 0] = 0.9
    c3, sc3 = O.uq_rowmax(big, 8, quantized=m)
    assert np.all(c3[:, [0, 5]] == 0)
    assert np.array_equal(sc3, (big[:, m].astype(np.float32).max(axis=1) / np.float32(255)).astype(np.float32))
    # a row of zeros: scale 1, codes 0
    cz, sz = O.uq_rowmax(np.zeros((2, 5)), 8)
    assert np.all(cz == 0) and np.all(sz == 1)
    # exact rational rounding on fp16-valued rows (products and quotients exact enough to decide every code)
    q = (rng.uniform(0, 1, size=(6, 40))).astype(np.float16)
    cq, _ = O.uq_rowmax(q.astype(np.float32), 8)
    for r in range(6):
        fr = [Fraction(float(v)) for v in q[r]]
        amax = max(fr)
        assert list(cq[r]) == [brute.round_half_even(v * 255 / amax) for v in fr]
