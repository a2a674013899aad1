"""Pins for the CPU oracle (no GPU).

The oracle is checked against what the paper and the mathematics fix, never
against itself: the Eq. 1 value table, brute force over all codes, a library
integer matmul on closed-form values, the XNOR-popcount special case, the
all-ones-matrix identity the paper quotes for prior work, and algebraic
invariants.  Each test names the mistake it is meant to catch.
"""
import itertools
import os

import numpy as np
import pytest

from paper_2409_17870_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bipolar_values.txt")


def closed_form(codes, n):
    """2u - (2^n - 1): the closed form of Eq. 1 (retyped here, not taken from the oracle)."""
    return 2 * codes.astype(np.int64) - ((1 << n) - 1)


def rand_codes(rng, rows, K, bits):
    return rng.integers(0, 1 << bits, size=(rows, K), dtype=np.uint8)


# ---------------------------------------------------------------- Eq. 1 ----
def test_value_table_matches_golden(oracle):
    """Sec. 3.1 Eq. 1 written out by hand for n = 1..4 (wrong sign / wrong weight per bit)."""
    with open(GOLDEN) as f:
        rows = [l for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for line in rows:
        n, vals = line.split(":")
        n = int(n)
        vals = [int(v) for v in vals.split()]
        assert len(vals) == 1 << n
        assert [oracle.bipolar_value(c, n) for c in range(1 << n)] == vals


@pytest.mark.parametrize("n", range(1, 9))
def test_value_closed_form_odd_symmetric(oracle, n):
    vals = np.array([oracle.bipolar_value(c, n) for c in range(1 << n)], dtype=np.int64)
    assert np.array_equal(vals, closed_form(np.arange(1 << n), n))
    assert np.all(vals % 2 != 0)                       # odd numbers only, no zero
    assert vals.min() == -((1 << n) - 1) and vals.max() == (1 << n) - 1
    assert np.array_equal(vals, -vals[::-1])           # symmetric range
    assert np.all(np.diff(vals) == 2)                  # monotone in the code


# ------------------------------------------------------- brute force ------
def test_single_products_all_codes(oracle):
    """K = 1, every (p, q) in 1..8 and every code pair: C = val(a) * val(w)."""
    for p in range(1, 9):
        for q in range(1, 9):
            a = np.arange(1 << p, dtype=np.uint8).reshape(-1, 1)
            w = np.arange(1 << q, dtype=np.uint8).reshape(-1, 1)
            want = np.outer(closed_form(a[:, 0], p), closed_form(w[:, 0], q))
            assert np.array_equal(oracle.gemm_i64(a, w, p, q), want), (p, q)
            assert np.array_equal(oracle.gemm_planes_i64(a, w, p, q), want), (p, q)


@pytest.mark.parametrize("p,q", [(1, 1), (1, 2), (2, 1), (2, 2)])
@pytest.mark.parametrize("K", [2, 3, 4])
def test_exhaustive_dot_products(oracle, p, q, K):
    """M = N = 1: every assignment of codes, python-loop dot product (dropped k term, wrong index)."""
    a_all = np.array(list(itertools.product(range(1 << p), repeat=K)), dtype=np.uint8)
    w_all = np.array(list(itertools.product(range(1 << q), repeat=K)), dtype=np.uint8)
    got = oracle.gemm_i64(a_all, w_all, p, q)
    got_planes = oracle.gemm_planes_i64(a_all, w_all, p, q)
    for ia, arow in enumerate(a_all):
        for iw, wrow in enumerate(w_all):
            s = 0
            for k in range(K):
                s += (2 * int(arow[k]) - ((1 << p) - 1)) * (2 * int(wrow[k]) - ((1 << q) - 1))
            assert got[ia, iw] == s
            assert got_planes[ia, iw] == s


# --------------------------------------------- library matmul special case --
@pytest.mark.parametrize("p,q", [(p, q) for p in range(1, 9) for q in range(1, 9)])
def test_against_numpy_matmul(oracle, p, q):
    """Ragged, non-square shapes, odd and even K (transposed operand, row/column mix-up)."""
    rng = np.random.default_rng(1000 * p + q)
    for (M, N, K) in [(3, 5, 7), (5, 2, 64), (1, 9, 33)]:
        a, w = rand_codes(rng, M, K, p), rand_codes(rng, N, K, q)
        want = closed_form(a, p) @ closed_form(w, q).T
        assert np.array_equal(oracle.gemm_i64(a, w, p, q), want)


@pytest.mark.parametrize("p,q", [(1, 1), (2, 1), (2, 2), (4, 1), (4, 2), (3, 4), (8, 8), (5, 7)])
def test_recovery_identity(oracle, p, q):
    """Sec. 3.2: planes + 1-bit products + shift-add recovery equals the value GEMM."""
    rng = np.random.default_rng(77 + 10 * p + q)
    for (M, N, K) in [(4, 6, 31), (7, 3, 96), (2, 2, 1)]:
        a, w = rand_codes(rng, M, K, p), rand_codes(rng, N, K, q)
        want = closed_form(a, p) @ closed_form(w, q).T
        assert np.array_equal(oracle.gemm_planes_i64(a, w, p, q), want)


def test_high_bits_of_codes_are_ignored(oracle):
    """Only the low `bits` bits of each byte are significant."""
    rng = np.random.default_rng(5)
    a, w = rand_codes(rng, 4, 20, 3), rand_codes(rng, 5, 20, 2)
    dirty_a = a | (rng.integers(0, 32, size=a.shape, dtype=np.uint8) << 3).astype(np.uint8)
    dirty_w = w | (rng.integers(0, 64, size=w.shape, dtype=np.uint8) << 2).astype(np.uint8)
    assert np.array_equal(oracle.gemm_i64(dirty_a, dirty_w, 3, 2), oracle.gemm_i64(a, w, 3, 2))
    assert np.array_equal(oracle.gemm_planes_i64(dirty_a, dirty_w, 3, 2), oracle.gemm_i64(a, w, 3, 2))


# ---------------------------------------------------------- special cases ---
def test_binary_case_is_xnor_popcount(oracle):
    """p = q = 1 is the textbook +-1 GEMM: C = K - 2 popcount(a xor w) on packed bits."""
    rng = np.random.default_rng(11)
    M, N, K = 6, 9, 200
    a, w = rand_codes(rng, M, K, 1), rand_codes(rng, N, K, 1)
    pa, pw = np.packbits(a, axis=1), np.packbits(w, axis=1)
    pop = np.array([[int(np.unpackbits(pa[m] ^ pw[n]).sum()) for n in range(N)] for m in range(M)])
    assert np.array_equal(oracle.gemm_i64(a, w, 1, 1), K - 2 * pop)


@pytest.mark.parametrize("p", [1, 2, 4])
def test_all_ones_matrix_identity(oracle, p):
    """Sec. 3.1: with 0/1-decoded binary weights W^, W = 2 W^ - J, so A W^T = 2 A W^^T - A J^T."""
    rng = np.random.default_rng(13 + p)
    M, N, K = 5, 7, 50
    a, w = rand_codes(rng, M, K, p), rand_codes(rng, N, K, 1)
    av = closed_form(a, p)
    w_hat = w.astype(np.int64)
    J = np.ones_like(w_hat)
    assert np.array_equal(oracle.gemm_i64(a, w, p, 1), 2 * (av @ w_hat.T) - av @ J.T)


# -------------------------------------------------------------- invariants --
@pytest.mark.parametrize("p,q", [(2, 1), (2, 2), (4, 2), (3, 5)])
def test_invariants(oracle, p, q):
    rng = np.random.default_rng(31 * p + q)
    M, N, K = 6, 4, 45
    a, w = rand_codes(rng, M, K, p), rand_codes(rng, N, K, q)
    c = oracle.gemm_i64(a, w, p, q)
    # a sum of K odd products has the parity of K
    assert np.all((c - K) % 2 == 0)
    # bound, attained by all-ones x all-ones (+) and all-ones x all-zeros (-)
    bound = K * ((1 << p) - 1) * ((1 << q) - 1)
    assert np.all(np.abs(c) <= bound)
    ones_a = np.full((1, K), (1 << p) - 1, dtype=np.uint8)
    ones_w = np.full((1, K), (1 << q) - 1, dtype=np.uint8)
    zeros_w = np.zeros((1, K), dtype=np.uint8)
    assert oracle.gemm_i64(ones_a, ones_w, p, q)[0, 0] == bound
    assert oracle.gemm_i64(ones_a, zeros_w, p, q)[0, 0] == -bound
    # complementing every bit of A negates C
    a_bar = (~a) & np.uint8((1 << p) - 1)
    assert np.array_equal(oracle.gemm_i64(a_bar, w, p, q), -c)
    # swapping the roles of the operands transposes C
    assert np.array_equal(oracle.gemm_i64(w, a, q, p), c.T)


def test_plane_linearity(oracle):
    """W1A2 = 2 * W1A1(activation plane 1) + W1A1(activation plane 0)."""
    rng = np.random.default_rng(3)
    a, w = rand_codes(rng, 5, 40, 2), rand_codes(rng, 6, 40, 1)
    c = oracle.gemm_i64(a, w, 2, 1)
    c0 = oracle.gemm_i64(a & 1, w, 1, 1)
    c1 = oracle.gemm_i64((a >> 1) & 1, w, 1, 1)
    assert np.array_equal(c, 2 * c1 + c0)


def test_gemm_i32_rejects_overflow(oracle):
    K = 40000                                   # 40000 * 255 * 255 > 2^31 - 1
    a = np.full((1, K), 255, dtype=np.uint8)
    w = np.full((1, K), 255, dtype=np.uint8)
    with pytest.raises(OverflowError):
        oracle.gemm_i32(a, w, 8, 8)
    assert oracle.gemm_i64(a, w, 8, 8)[0, 0] == K * 255 * 255


def test_empty_shapes(oracle):
    a = np.zeros((0, 8), dtype=np.uint8)
    w = np.zeros((3, 8), dtype=np.uint8)
    assert oracle.gemm_i64(a, w, 2, 2).shape == (0, 3)
    assert oracle.gemm_i64(w, a, 2, 2).shape == (3, 0)


# ---------------------------------------------------------------- epilogue --
def test_half_decode_all_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_bits_to_double(int(b)) for b in bits])
    finite = np.isfinite(want)
    assert np.array_equal(got[finite], want[finite])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))
    assert np.array_equal(np.signbit(got[~np.isnan(want)]), np.signbit(want[~np.isnan(want)]))


def test_scale_epilogue(oracle):
    rng = np.random.default_rng(21)
    c = rng.integers(-600000, 600000, size=(5, 7), dtype=np.int64)
    sa = rng.uniform(0.01, 0.1, 5).astype(np.float16)
    sw = rng.uniform(0.01, 0.1, 7).astype(np.float16)
    want = c.astype(np.float64) * sa.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :]
    got = oracle.scale_f64(c, sa.view(np.uint16), sw.view(np.uint16))
    assert np.allclose(got, want, rtol=1e-15, atol=0)
    assert np.array_equal(oracle.scale_f64(c), c.astype(np.float64))
    only_w = oracle.scale_f64(c, None, sw.view(np.uint16))
    assert np.allclose(only_w, c * sw.astype(np.float64)[None, :], rtol=1e-15, atol=0)


# --------------------------------------------------- generator sanity -------
def test_generator_reproducible_and_balanced():
    a1 = inputs.bernoulli_codes(inputs.BASE_SEED + 2, inputs.TAG_A, 64, 256, 2)
    a2 = inputs.bernoulli_codes(inputs.BASE_SEED + 2, inputs.TAG_A, 64, 256, 2)
    assert np.array_equal(a1, a2) and a1.max() <= 3
    for b in range(2):
        frac = ((a1 >> b) & 1).mean()
        assert abs(frac - 0.5) < 0.02
    w = inputs.bernoulli_codes(inputs.BASE_SEED + 2, inputs.TAG_W, 64, 256, 1)
    assert not np.array_equal(w, a1 & 1)
    n = inputs.normal_codes(7, inputs.TAG_A, 128, 256, bits=4)
    assert n.min() >= 0 and n.max() <= 15
    assert abs(n.astype(np.float64).mean() - 7.5) < 0.1       # centred on the middle of the range
    s = inputs.scales_f16(7, inputs.TAG_W_SCALE, 1000)
    assert s.dtype == np.float16 and s.min() >= 0.01 and s.max() <= 0.1


def test_result_statistics_of_bernoulli_inputs(oracle):
    """i.i.d. Bernoulli(1/2) bits give E[C] = 0 and Var[C] = K (4^p - 1)(4^q - 1) / 9."""
    p, q, K = 2, 1, 512
    a = inputs.bernoulli_codes(99, inputs.TAG_A, 64, K, p)
    w = inputs.bernoulli_codes(99, inputs.TAG_W, 64, K, q)
    c = oracle.gemm_i64(a, w, p, q).astype(np.float64)
    var = K * (4 ** p - 1) * (4 ** q - 1) / 9.0
    assert abs(c.mean()) < 4 * np.sqrt(var / c.size) + 1.0
    assert 0.85 * var < c.var() < 1.15 * var


def test_config_cases_cover_the_five_workloads():
    shapes = {i: inputs.config_cases(i) for i in range(1, 6)}
    assert shapes[1][0] == dict(M=16, N=256, K=512, p=2, q=1, a_dist="bernoulli", scaled=False)
    assert (shapes[2][0]["M"], shapes[2][0]["N"], shapes[2][0]["K"]) == (4096, 4096, 4096)
    assert len(shapes[3]) == 9 and len(shapes[4]) == 6 and len(shapes[5]) == 7
    case = inputs.make_case(dict(M=2, N=3, K=64, p=4, q=2, a_dist="normal", scaled=True), 5)
    assert case["a_codes"].shape == (2, 64) and case["w_codes"].shape == (3, 64)
    assert case["a_scale"].shape == (2,) and case["w_scale"].shape == (3,)


# --------------------------------------------- quantisation onto the grid --
def _val(codes, p):
    return 2 * codes.astype(np.int64) - ((1 << p) - 1)


def test_float_to_half_matches_the_library_conversion(oracle):
    """The oracle's own binary32 -> binary16 rounding against numpy's, including subnormals,
    ties and the overflow threshold."""
    rng = np.random.default_rng(11)
    vals = [rng.normal(size=3000).astype(np.float32) * np.float32(s) for s in (1e-8, 1e-6, 1e-4, 1e-2, 1, 100, 30000)]
    ties = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -25, 3 * 2.0 ** -25, 2.0 ** -24, 65504.0, 65519.0,
                     65520.0, 0.0, -0.0, 6.1e-5, -2.5], dtype=np.float32)
    with np.errstate(over="ignore"):
        for v in np.concatenate(vals + [ties]):
            assert oracle.float_to_half_bits(v) == int(np.float32(v).astype(np.float16).view(np.uint16)), v


def _golden_quantize_rows():
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "quantize_borders.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p, s, x, c = [t.strip() for t in line.split(":")]
            rows.append((int(p), int(s, 16), np.array([int(t, 16) for t in x.split()], dtype=np.uint16),
                         np.array([int(t) for t in c.split()], dtype=np.uint8)))
    return rows


def test_quantize_matches_the_hand_worked_border_rows(oracle):
    """Sec. 3.1 quantiser on rows with non-power-of-two scales and elements on, just below and just above
    cell borders; scale and codes worked by hand in tests/golden/quantize_borders.txt.  (A quantiser that
    multiplies by a rounded reciprocal of the scale lands in the lower cell at 4 s and 8 s of the third row.)"""
    rows = _golden_quantize_rows()
    assert [r[0] for r in rows] == [2, 3, 4]
    for p, sbits, xbits, want in rows:
        codes, s = oracle.quantize_rows(xbits.view(np.float16).reshape(1, -1), p)
        assert int(s[0]) == sbits
        assert np.array_equal(codes[0], want), (p, codes[0], want)


def _nearest_odd_code(x, s, p):
    """Code of the grid point nearest to x / s in exact rational arithmetic: argmin over all 2^p grid
    values of |x / s - v|, the larger v on a tie."""
    from fractions import Fraction
    t = Fraction(float(x)) / Fraction(float(s))
    best = None
    for u in range(1 << p):
        d = abs(t - (2 * u - ((1 << p) - 1)))
        if best is None or d <= best[0]:
            best = (d, u)
    return best[1]


@pytest.mark.parametrize("p", [1, 2, 3, 4, 6, 8])
def test_quantize_is_the_nearest_grid_point_in_exact_arithmetic(oracle, p):
    """Brute force from the definition: for rows with arbitrary (non-power-of-two) scales, every element
    gets the code whose grid value is nearest to x / s, compared as exact fractions.  The rows hold random
    values plus, for every border of the grid, the binary16 numbers at and around border * s."""
    top = (1 << p) - 1
    rng = np.random.default_rng(100 + p)
    for trial in range(12):
        amax = np.float16(rng.uniform(0.01, 900.0) if trial else 6.1e-5 * 3)   # one row with a subnormal scale
        s_guess = np.float16(np.float32(amax) / np.float32(top))
        extra = []
        for c in range(1, top + 1):
            b = np.float16(np.float64(2 * c - (1 << p)) * np.float64(s_guess))
            for step in (-2, -1, 0, 1, 2):
                v = (b.view(np.int16) + np.int16(step)).view(np.float16) if b != 0 else np.float16(step * 6e-8)
                if np.isfinite(v) and abs(float(v)) <= float(amax):
                    extra.append(v)
        rnd = (rng.normal(size=40) * float(amax) / 2.5).astype(np.float16)
        rnd = rnd[np.abs(rnd.astype(np.float64)) <= float(amax)]
        x = np.concatenate([[amax], np.array(extra, dtype=np.float16), rnd]).astype(np.float16)
        codes, sb = oracle.quantize_rows(x.reshape(1, -1), p)
        s = sb.view(np.float16)[0]
        # the scale: exact quotient, one rounding to binary16 (numpy rounds the exact double quotient's
        # float32 rounding; both agree, see the oracle's note on ties)
        from fractions import Fraction
        q = Fraction(float(amax)) / top
        lo, hi = np.nextafter(s, np.float16(-np.inf)), np.nextafter(s, np.float16(np.inf))
        assert abs(Fraction(float(s)) - q) <= abs(Fraction(float(lo)) - q)
        assert abs(Fraction(float(s)) - q) <= abs(Fraction(float(hi)) - q)
        assert s > 0
        want = np.array([_nearest_odd_code(v, s, p) for v in x], dtype=np.uint8)
        assert np.array_equal(codes[0], want), (p, trial)


def test_double_to_half_is_one_rounding(oracle):
    """double -> binary16 directly, not through binary32: values chosen so that rounding to binary32 first
    would land on a binary16 tie and then go the other way."""
    x = 1.0 + 2.0 ** -11 + 2.0 ** -30           # just above the tie between 1 and 1 + 2^-10
    assert np.float32(x) == np.float32(1.0 + 2.0 ** -11)       # binary32 loses the 2^-30
    assert oracle.double_to_half_bits(x) == 0x3C01              # the exact value rounds up
    assert oracle.double_to_half_bits(1.0 + 2.0 ** -11) == 0x3C00   # the tie itself goes to even
    assert oracle.double_to_half_bits(1.0 + 3 * 2.0 ** -11 - 2.0 ** -30) == 0x3C01
    assert oracle.double_to_half_bits(1e300) == 0x7C00 and oracle.double_to_half_bits(-1e300) == 0xFC00
    assert oracle.double_to_half_bits(65519.999) == 0x7BFF and oracle.double_to_half_bits(65520.0) == 0x7C00


def test_quantize_one_bit_is_the_sign(oracle):
    """Sec. 3.1: 1-bit bipolar-INT is binary quantisation, code = [x >= 0], scale = max|x|."""
    x = inputs.normal_features_f16(21, inputs.TAG_A, 9, 200)
    codes, scale = oracle.quantize_rows(x, 1)
    assert np.array_equal(codes, (x >= 0).astype(np.uint8))
    assert np.array_equal(scale.view(np.float16), np.abs(x).max(axis=1))


@pytest.mark.parametrize("p", [2, 3, 4, 8])
def test_quantize_is_exact_on_the_grid(oracle, p):
    """Features that already are scale * (odd integers of the grid) come back as their own codes."""
    top = (1 << p) - 1
    rng = np.random.default_rng(p)
    for scale in (2.0 ** -3, 2.0 ** -10, 1.0):
        want = rng.integers(0, top + 1, size=(6, 77)).astype(np.uint8)
        want[:, 0] = top                                  # the row maximum fixes the scale
        if scale * top > 65504:
            continue
        x = (scale * _val(want, p)).astype(np.float16)
        codes, s = oracle.quantize_rows(x, p)
        assert np.array_equal(codes, want)
        assert np.all(s.view(np.float16) == np.float16(scale))


@pytest.mark.parametrize("p", [2, 3, 4, 5])
def test_quantize_properties(oracle, p):
    """Nearest grid point: |x - s val(u)| <= s unless clamped; the row maximum takes an outermost code;
    codes never decrease with x; a zero row has scale 0 and the code of +1."""
    top = (1 << p) - 1
    x = inputs.normal_features_f16(30 + p, inputs.TAG_A, 40, 333, outlier_every=50)
    x[7] = 0
    codes, sbits = oracle.quantize_rows(x, p)
    s = sbits.view(np.float16).astype(np.float64)
    xd = x.astype(np.float64)
    err = np.abs(xd - s[:, None] * _val(codes, p))
    inside = np.abs(xd) <= s[:, None] * top
    assert np.all(err[inside] <= s[:, None].repeat(x.shape[1], 1)[inside] * (1 + 1e-6))
    rows = np.arange(x.shape[0])
    at_max = codes[rows, np.abs(xd).argmax(axis=1)]
    nz = s > 0
    assert np.all((at_max[nz] == top) | (at_max[nz] == 0))
    for m in range(x.shape[0]):
        order = np.argsort(xd[m], kind="stable")
        assert np.all(np.diff(codes[m, order].astype(np.int64)) >= 0)
    assert sbits[7] == 0 and np.all(codes[7] == 1 << (p - 1))
    want_scale = (np.abs(x.astype(np.float32)).max(axis=1) / np.float32(top)).astype(np.float16)
    assert np.array_equal(sbits, want_scale.view(np.uint16))


def test_quantize_brute_force_all_halves(oracle):
    """Every finite binary16 value in one row with a power-of-two scale: the code is the cell of width 2
    (in units of the scale) that holds the value, counted from the bottom of the grid."""
    p, top = 3, 7
    bits = np.arange(0x10000, dtype=np.uint16)
    x = bits.view(np.float16)
    x = x[np.isfinite(x) & (np.abs(x.astype(np.float64)) <= 7 * 0.25)]      # max |x| = 1.75 -> scale 0.25
    codes, s = oracle.quantize_rows(x.reshape(1, -1), p)
    assert s.view(np.float16)[0] == np.float16(0.25)
    t = x.astype(np.float64) / 0.25                                          # exact
    want = np.clip(np.floor(t / 2.0) + 4, 0, top).astype(np.uint8)
    assert np.array_equal(codes[0], want)

