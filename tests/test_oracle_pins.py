"""Pins for the CPU oracle: every check here compares the oracle with something
other than itself - values derived by hand from Eq. 1-7 (tests/golden/), closed
forms, invariants of the Hadamard matrix, brute force in exact integers, or an
fp64 computation of the un-quantised product."""
import math

import numpy as np
import pytest

from oracle import hbl_oracle as O
from paper_2504_18415_amd import synth

EPS = 1e-5


def popcount_hadamard(n):
    """Closed form of Eq. 4: H[i][j] = (-1)^popcount(i & j) / sqrt(n)."""
    i = np.arange(n)
    a = i[:, None] & i[None, :]
    pc = np.zeros_like(a)
    while a.any():
        pc += a & 1
        a >>= 1
    return np.where(pc % 2 == 0, 1.0, -1.0) / math.sqrt(n)


# ---------------------------------------------------------------- Eq. 3-4
@pytest.mark.parametrize("m", [0, 1, 2, 3, 4, 5, 6])
def test_dense_hadamard_orthogonal_and_closed_form(m):
    n = 1 << m
    H = O.hadamard_dense(m)
    assert np.allclose(H @ H.T, np.eye(n), atol=1e-12)          # orthogonality, fixes 1/sqrt(2) per level
    assert np.allclose(H, H.T, atol=0)                            # symmetric
    assert np.allclose(H, popcount_hadamard(n), atol=1e-12)      # Sylvester / natural ordering


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64])
def test_fwht_equals_dense_matmul(n):
    rng = np.random.default_rng(n)
    x = rng.standard_normal((5, n)).astype(np.float32)
    ref = x.astype(np.float64) @ popcount_hadamard(n)            # rows: x H (H symmetric)
    got = O.fwht_rows(x)
    assert np.allclose(got, ref, rtol=0, atol=4e-6 * np.abs(x).sum(axis=1, keepdims=True) / math.sqrt(n) + 1e-7)
    # and against the recursion-built matrix of the oracle itself
    assert np.allclose(got, x.astype(np.float64) @ O.hadamard_dense(int(math.log2(n))), atol=1e-5)


@pytest.mark.parametrize("n", [256, 2048, 4096, 8192, 16384])
def test_fwht_exact_on_small_integers_at_full_size(n):
    """Integer inputs keep every partial sum an integer below 2^24, so fp32 butterflies are exact;
    compare c_n * (integer closed form) on sampled output indices."""
    rng = np.random.default_rng(100 + n)
    x = rng.integers(-7, 8, size=(3, n)).astype(np.float32)
    got = O.fwht_rows(x)
    c_n = np.float32(1.0 / math.sqrt(n))
    idx = np.concatenate([[0, 1, 2, n // 2, n - 1], rng.integers(0, n, 40)])
    j = np.arange(n)
    for i in idx:
        pc = np.array([bin(int(i) & int(v)).count("1") & 1 for v in j])
        row = np.where(pc == 0, 1, -1).astype(np.int64)
        exact = (x.astype(np.int64) * row).sum(axis=1)
        assert np.all(np.abs(exact) < 2 ** 24)
        want = exact.astype(np.float32) * c_n
        assert np.array_equal(got[:, i], want), (n, i)


@pytest.mark.parametrize("n", [16, 512, 4096])
def test_fwht_invariants(n):
    rng = np.random.default_rng(7)
    x = rng.standard_normal((4, n)).astype(np.float32)
    y = O.fwht_rows(x)
    # Parseval
    assert np.allclose((y.astype(np.float64) ** 2).sum(1), (x.astype(np.float64) ** 2).sum(1), rtol=1e-5)
    # involution (orthogonal + symmetric)
    assert np.allclose(O.fwht_rows(y), x, atol=2e-5)
    # unit vector e_j -> column j; all-ones -> sqrt(n) e_0
    j = 5 % n
    e = np.zeros((1, n), np.float32)
    e[0, j] = 1
    assert np.allclose(O.fwht_rows(e)[0], popcount_hadamard(n)[:, j] if n <= 512 else
                       np.array([(-1) ** bin(i & j).count("1") for i in range(n)]) / math.sqrt(n), atol=1e-7)
    ones = np.ones((1, n), np.float32)
    t = O.fwht_rows(ones)[0]
    assert abs(t[0] - math.sqrt(n)) < 1e-4 and np.all(t[1:] == 0)


def test_fwht_normalisation_constants():
    """c_n is an exact power of two for even m and a rounded 1/sqrt(n) otherwise."""
    for n, want in [(256, 2.0 ** -4), (4096, 2.0 ** -6), (16384, 2.0 ** -7)]:
        e = np.zeros((1, n), np.float32)
        e[0, 0] = 1
        assert O.fwht_rows(e)[0, 0] == np.float32(want)
    for n in (2048, 8192):
        e = np.zeros((1, n), np.float32)
        e[0, 0] = 1
        assert O.fwht_rows(e)[0, 0] == np.float32(1.0 / math.sqrt(n))


# ---------------------------------------------------------------- hand examples
def test_hand_example_hadamard_then_quant(golden):
    g = golden["hadamard_quant_n4"]
    x = np.array([g["x"]], np.float32)
    assert np.array_equal(O.fwht_rows(x)[0], np.array(g["x_r"], np.float32))
    c8, s8, xr = O.fwht_quant(x, 8, hadamard=True, eps=g["eps"][0], want_xr=True)
    assert np.array_equal(xr[0], np.array(g["x_r"], np.float32))
    assert c8[0].tolist() == g["codes_int8"]
    assert s8[0] == np.float32(g["s_dequant_int8"][0])
    c4, s4 = O.fwht_quant(x, 4, hadamard=True, eps=g["eps"][0])
    assert c4[0].tolist() == g["codes_int4"]
    assert abs(float(s4[0]) - g["s_dequant_int4"][0]) <= 6e-8


def test_hand_example_ternarize(golden):
    g = golden["ternarize_2x2"]
    codes, alpha = O.ternarize_weights_absmean(np.array(g["w"], np.float32).reshape(2, 2), g["eps"][0])
    assert codes.reshape(-1).tolist() == g["codes"]
    assert abs(float(alpha) - g["alpha"][0]) < 1e-7


def test_hand_example_ties_half_even(golden):
    g = golden["int8_ties_half_even"]
    c, s = O.fwht_quant(np.array([g["x"]], np.float32), 8, hadamard=False, eps=0.0)
    assert c[0].tolist() == g["codes_int8"] and s[0] == np.float32(1.0)


def test_hand_example_int4_clip(golden):
    g = golden["int4_clip_asymmetric"]
    c, s = O.fwht_quant(np.array([g["x"]], np.float32), 4, hadamard=False, eps=g["eps"][0])
    assert c[0].tolist() == g["codes_int4"]
    assert abs(float(s[0]) - g["s_dequant_int4"][0]) < 2e-7


def test_hand_example_eps_placement(golden):
    g = golden["int8_eps_placement"]
    c, s = O.fwht_quant(np.array([g["x"]], np.float32), 8, hadamard=False, eps=g["eps"][0])
    assert c[0].tolist() == g["codes_int8"]
    assert abs(float(s[0]) / g["s_dequant_int8"][0] - 1) < 1e-6


def test_hand_example_int8_clip_bounds(golden):
    g = golden["int8_clip_bounds_negative_eps"]
    c, s = O.fwht_quant(np.array([g["x"]], np.float32), 8, hadamard=False, eps=g["eps"][0])
    assert c[0].tolist() == g["codes_int8"]
    assert s[0] == np.float32(g["s_dequant_int8"][0])


# ---------------------------------------------------------------- Eq. 5-6 invariants
@pytest.mark.parametrize("hadamard", [False, True])
def test_quantizer_ranges_and_boundaries(hadamard):
    site = synth.config_sites(1)[0]
    x = synth.make_x(site)
    c8, s8, xr = O.fwht_quant(x, 8, hadamard=hadamard, want_xr=True)
    assert c8.min() >= -127 and c8.max() <= 127                 # |127 x/(gamma+eps)| < 127
    am = np.abs(xr).argmax(axis=1)
    assert np.all(np.abs(c8[np.arange(len(am)), am]) == 127)     # the arg-max element maps to +-127
    assert np.allclose(s8 * 127, np.abs(xr).max(1), rtol=1e-6)
    c4, s4 = O.fwht_quant(x, 4, hadamard=hadamard)
    assert c4.min() >= -8 and c4.max() <= 7
    assert np.allclose(s4 * math.sqrt(7), np.abs(xr.astype(np.float64)).mean(1), rtol=1e-6)
    # reconstruction: unclipped entries are within half a step
    for c, s, lo, hi in ((c8, s8, -128, 127), (c4, s4, -8, 7)):
        unclipped = (c > lo) & (c < hi)
        step = (s * (1 + 2e-5))[:, None]          # gain uses +eps, the outer factor does not
        err = np.abs(xr - c * s[:, None])
        assert np.all(err[unclipped] <= (0.5 * step + 1e-6 * np.abs(xr))[unclipped] + 2e-5 * np.abs(xr)[unclipped])


def test_zero_row_gives_zero_codes_and_finite_scales():
    x = np.zeros((2, 64), np.float32)
    for bits in (4, 8):
        c, s = O.fwht_quant(x, bits, hadamard=True)
        assert not c.any() and np.all(s == 0) and np.all(np.isfinite(s))
    wc = np.ones((8, 64), np.int8)
    y = O.hbitlinear_forward(x, wc, np.float32(0.5), 4)
    assert not y.any()


def test_gaussian_closed_forms():
    """x ~ N(0,1): beta -> sqrt(2/pi), clip fractions of Eq. 6; W ~ N(0,0.02^2): alpha -> 0.7979 sigma,
    P(code != 0) = 2(1 - Phi(0.5 * 0.7979))."""
    from scipy.stats import norm
    rng = np.random.default_rng(3)
    x = rng.standard_normal((64, 16384)).astype(np.float32)
    c4, s4 = O.fwht_quant(x, 4, hadamard=False)
    beta = s4.astype(np.float64) * math.sqrt(7)
    assert np.allclose(beta, math.sqrt(2 / math.pi), rtol=0.03)
    gain = math.sqrt(7) / math.sqrt(2 / math.pi)
    p_hi = 1 - norm.cdf(6.5 / gain)      # rounds to >= 7
    p_lo = norm.cdf(-7.5 / gain)         # rounds to <= -8
    assert abs((c4 == 7).mean() - p_hi) < 0.1 * p_hi
    assert abs((c4 == -8).mean() - p_lo) < 0.1 * p_lo
    W = (rng.standard_normal((512, 2048)) * 0.02).astype(np.float32)
    codes, alpha = O.ternarize_weights_absmean(W)
    assert abs(alpha - 0.02 * math.sqrt(2 / math.pi)) < 2e-4
    assert alpha == np.float32(np.abs(W.astype(np.float64)).mean())
    assert set(np.unique(codes)) == {-1, 0, 1}
    p_nz = 2 * (1 - norm.cdf(0.5 * math.sqrt(2 / math.pi)))
    assert abs((codes != 0).mean() - p_nz) < 0.01
    assert abs((codes == 1).mean() - (codes == -1).mean()) < 0.01
    # codes agree with the definition evaluated in fp64 except within rounding distance of a boundary
    r = W.astype(np.float64) / (float(alpha) + 1e-5)
    want = np.clip(np.rint(r), -1, 1)
    near = np.abs(np.abs(r) - 0.5) < 1e-5
    assert np.array_equal(codes[~near], want[~near].astype(np.int8))


def test_bf16_input_equals_widened_fp32_input():
    site = synth.shrink(synth.config_sites(2)[0], T=8, K=256)
    xb = synth.make_x(site)
    xf = synth.bf16_bits_to_f32(xb)
    for bits in (4, 8):
        cb, sb = O.fwht_quant(xb, bits)
        cf, sf = O.fwht_quant(xf, bits)
        assert np.array_equal(cb, cf) and np.array_equal(sb, sf)
    # the widening itself: 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCD ~ 0.1001
    assert synth.bf16_bits_to_f32(np.array([0x3F80, 0xC000], np.uint16)).tolist() == [1.0, -2.0]
    c, _ = O.fwht_quant(np.array([[0x3F80, 0xC000]], np.uint16), 8, hadamard=False)
    assert c[0].tolist() == [63, -127]   # 127/(2+1e-5) = 63.4997 -> 63; times -2 = -126.9994 -> -127


# ---------------------------------------------------------------- integer GEMM
def test_gemm_brute_force_tiny():
    rng = np.random.default_rng(11)
    for (T, K, N) in [(1, 1, 1), (3, 5, 2), (4, 16, 7), (2, 33, 3)]:
        q = rng.integers(-128, 128, (T, K)).astype(np.int8)
        c = rng.integers(-1, 2, (N, K)).astype(np.int8)
        want = [[sum(int(q[t, k]) * int(c[o, k]) for k in range(K)) for o in range(N)] for t in range(T)]
        assert O.gemm_i32(q, c).tolist() == want


def test_gemm_vs_int64_matmul_and_identity():
    rng = np.random.default_rng(12)
    q = rng.integers(-128, 128, (37, 512)).astype(np.int8)
    c = rng.integers(-1, 2, (29, 512)).astype(np.int8)
    assert np.array_equal(O.gemm_i32(q, c), q.astype(np.int64) @ c.astype(np.int64).T)
    eye = np.eye(512, dtype=np.int8)
    assert np.array_equal(O.gemm_i32(q, eye), q.astype(np.int32))
    # extreme magnitudes stay exact in int32
    qm = np.full((2, 16384), -128, np.int8)
    cm = np.full((3, 16384), -1, np.int8)
    assert np.all(O.gemm_i32(qm, cm) == 128 * 16384)


# ---------------------------------------------------------------- epilogue / Eq. 7
def test_dequant_rounding_to_bf16_is_nearest_even():
    acc = np.array([[1, 1, 1, 3, -1]], np.int32)
    sd = np.array([1.0], np.float32)
    # one scale group per column so that each product is set independently
    a = np.array([1 + 2 ** -8, 1 + 3 * 2 ** -8, 1 + 2 ** -8 + 2 ** -20, 0.5, 1 + 2 ** -8], np.float32)
    y = O.dequant_bf16(acc, sd, a)
    got = synth.bf16_bits_to_f32(y)[0].tolist()
    assert got == [1.0, 1 + 2 ** -6, 1 + 2 ** -7, 1.5, -1.0]


def test_dequant_group_scales_and_token_scales():
    acc = np.arange(1, 13, dtype=np.int32).reshape(2, 6)
    sd = np.array([0.5, 2.0], np.float32)
    al = np.array([1.0, 4.0, 0.25], np.float32)     # three groups of two output rows
    y = synth.bf16_bits_to_f32(O.dequant_bf16(acc, sd, al))
    want = acc * sd[:, None] * np.repeat(al, 2)[None, :]
    assert np.array_equal(y, want.astype(np.float32))


def test_identity_weight_hand_case(golden):
    """W = I_4: alpha = 1/4, codes = I, so y[o] = bf16(q[o] * s_d * alpha) on the hand example row."""
    g = golden["hadamard_quant_n4"]
    x = np.array([g["x"]], np.float32)
    wc, alpha = O.ternarize_weights_absmean(np.eye(4, dtype=np.float32))
    assert alpha == np.float32(0.25) and np.array_equal(wc, np.eye(4, dtype=np.int8))
    y = synth.bf16_bits_to_f32(O.hbitlinear_forward(x, wc, alpha, 8))[0]
    want = np.array(g["codes_int8"]) * (5.0 / 127.0) * 0.25
    assert np.allclose(y, want, rtol=2 ** -8)
    y4 = synth.bf16_bits_to_f32(O.hbitlinear_forward(x, wc, alpha, 4))[0]
    assert np.allclose(y4, np.array(g["codes_int4"]) * (2 / math.sqrt(7)) * 0.25, rtol=2 ** -8)


def _float_reference(x_f32, W, hadamard):
    """alpha * codes_W . (H x) in fp64 with no activation quantisation."""
    wc, alpha = O.ternarize_weights_absmean(W)
    xr = x_f32.astype(np.float64)
    if hadamard:
        n = xr.shape[1]
        xr = xr @ popcount_hadamard(n)
    return (xr @ wc.astype(np.float64).T) * float(alpha), wc, alpha


@pytest.mark.parametrize("bits,bound", [(8, 0.02), (4, 0.15)])
def test_forward_close_to_unquantised_product(bits, bound):
    site = synth.shrink(synth.config_sites(2)[0], T=24, K=1024, N=96)
    xb = synth.make_x(site)
    W = synth.make_w(site)
    ref, wc, alpha = _float_reference(synth.bf16_bits_to_f32(xb), W, True)
    y = synth.bf16_bits_to_f32(O.hbitlinear_forward(xb, wc, alpha, bits)).astype(np.float64)
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert rel < bound, rel
    assert rel > 1e-4            # it IS quantised
    # plain path against the un-rotated product
    ref_p, _, _ = _float_reference(synth.bf16_bits_to_f32(xb), W, False)
    yp = synth.bf16_bits_to_f32(O.plain_bitlinear_forward(xb, wc, alpha, 8)).astype(np.float64)
    assert np.linalg.norm(yp - ref_p) / np.linalg.norm(ref_p) < 0.25


def test_scale_covariance():
    site = synth.shrink(synth.config_sites(2)[0], T=4, K=512, N=32)
    x = synth.bf16_bits_to_f32(synth.make_x(site))
    W = synth.make_w(site)
    wc, alpha = O.ternarize_weights_absmean(W)
    y1, c1, s1, a1 = O.hbitlinear_forward(x, wc, alpha, 8, want_intermediates=True)
    y2, c2, s2, a2 = O.hbitlinear_forward(2 * x, wc, alpha, 8, want_intermediates=True)
    assert (c1 != c2).mean() < 1e-3 and np.abs(c1.astype(int) - c2).max() <= 1
    assert np.allclose(s2, 2 * s1, rtol=1e-6)


def test_hadamard_removes_outlier_damage():
    """Section 2.1's claim on config-1 inputs: after the transform the row is Gaussian-like
    (small excess kurtosis) and INT4 reconstruction error drops."""
    site = synth.config_sites(1)[0]
    x = synth.make_x(site)

    def stats(hadamard):
        c, s, xr = O.fwht_quant(x, 4, hadamard=hadamard, want_xr=True)
        z = xr.astype(np.float64)
        kurt = ((z - z.mean(1, keepdims=True)) ** 4).mean(1) / z.var(1) ** 2 - 3
        mse = ((z - c * s[:, None].astype(np.float64)) ** 2).sum() / (z ** 2).sum()
        return kurt.mean(), mse

    k0, e0 = stats(False)
    k1, e1 = stats(True)
    assert k0 > 20 and abs(k1) < 1.5
    assert e1 < 0.25 * e0


# --- backward pass through the transform (Section 2.2, Eq. 8) -------------------------------------

@pytest.mark.parametrize("n", [16, 256, 4096])
def test_backward_adjoint_identity_on_exact_integers(n):
    """<Hadamard(x), y> = <x, backward(y)> must hold exactly when every value is a small integer and
    1/sqrt(n) a power of two (n a power of four): that is what "the gradient of the transform is the
    transform" means, and a transposed or unnormalised backward fails it."""
    rng = np.random.default_rng(n)
    x = rng.integers(-8, 9, size=(3, n)).astype(np.float32)
    y = rng.integers(-8, 9, size=(3, n)).astype(np.float32)
    hx = O.fwht_rows(x).astype(np.float64)
    by = O.hadamard_backward(y).astype(np.float64)
    assert np.array_equal((hx * y).sum(1), (x * by).sum(1))


@pytest.mark.parametrize("m", [1, 3, 6])
def test_backward_is_gradient_of_linear_functional(m):
    """L(x) = sum_i c_i * Hadamard(x)_i has dL/dx_j = sum_i c_i H[i][j]: the dense matrix (pinned on its
    own by H H^T = I and the popcount form) gives the gradient in fp64, central differences confirm it."""
    n = 1 << m
    rng = np.random.default_rng(100 + m)
    c = rng.standard_normal((1, n)).astype(np.float32)
    H = O.hadamard_dense(m).astype(np.float64)
    want = c.astype(np.float64) @ H                    # row vector times H = (H^T c)^T
    got = O.hadamard_backward(c).astype(np.float64)
    assert np.allclose(got, want, rtol=0, atol=4e-6 * np.abs(want).max())
    x0 = rng.standard_normal(n)
    L = lambda x: float((c[0].astype(np.float64) * (H @ x)).sum())
    for j in range(min(n, 8)):
        e = np.zeros(n)
        e[j] = 1e-3
        fd = (L(x0 + e) - L(x0 - e)) / 2e-3
        assert abs(fd - got[0, j]) <= 1e-5 * max(1.0, abs(fd))


def test_backward_undoes_forward_and_rounds_bf16_to_nearest_even():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((5, 1024)).astype(np.float32)
    back = O.hadamard_backward(O.fwht_rows(x))
    assert np.abs(back - x).max() <= 5e-6 * np.abs(x).max() * math.log2(1024)
    # bf16 in and out: equals widening, transforming in fp32 and an independent nearest-even narrowing
    xb = synth.f32_to_bf16_bits(x)
    want = synth.f32_to_bf16_bits(O.fwht_rows(synth.bf16_bits_to_f32(xb)))
    assert np.array_equal(O.hadamard_backward(xb, out_bf16=True), want)
    # a tie: 1 + 2^-8 is exactly half way between two bf16 values and must go to the even one (1.0)
    tie = np.zeros((1, 4), np.float32)
    tie[0, 0] = 2.0 * (1.0 + 2.0 ** -8)               # H_4 row sum / 2 keeps the value on entry 0..3
    out = synth.bf16_bits_to_f32(O.hadamard_backward(tie, out_bf16=True))
    assert np.array_equal(out, np.full((1, 4), 1.0, np.float32))


# --- LN of Eq. 7 as RMS normalisation ---------------------------------------------------------------

@pytest.mark.parametrize("case", ["rmsnorm_power_of_two", "rmsnorm_eps_placement"])
def test_rmsnorm_hand_examples(golden, case):
    c = golden[case]
    gain = np.array(c["gain"], np.float32)
    for i in range(2):
        if f"x{i}" not in c:
            continue
        x = np.array([c[f"x{i}"]], np.float32)
        got = O.rmsnorm(x, gain, c["ln_eps"][0])
        assert np.array_equal(got, np.array([c[f"y{i}"]], np.float32))
        got_b = O.rmsnorm(synth.f32_to_bf16_bits(x), gain, c["ln_eps"][0])      # bf16 input, same values
        assert np.array_equal(got_b, got)


def test_rmsnorm_invariants_and_fp64_reference():
    rng = np.random.default_rng(21)
    K = 1536                                           # not a power of two: the plain projections allow it
    x = (rng.standard_normal((9, K)) * rng.uniform(0.1, 30, (9, 1))).astype(np.float32)
    ones = np.ones(K, np.float32)
    y = O.rmsnorm(x, ones, 0.0).astype(np.float64)
    assert np.allclose((y ** 2).mean(1), 1.0, rtol=0, atol=2e-6)          # unit mean square
    # scaling a row by a power of two changes nothing when ln_eps = 0 (every step scales exactly)
    assert np.array_equal(O.rmsnorm(x * np.float32(8.0), ones, 0.0), O.rmsnorm(x, ones, 0.0))
    # gain multiplies element-wise; an fp64 evaluation of the definition agrees to fp32 rounding
    g = rng.standard_normal(K).astype(np.float32)
    eps = 1e-5
    want = x.astype(np.float64) / np.sqrt((x.astype(np.float64) ** 2).mean(1, keepdims=True) + eps) * g
    got = O.rmsnorm(x, g, eps)
    assert np.abs(got - want).max() <= 3e-7 * np.abs(want).max()
    assert np.abs(got - want).max() > 0                                    # fp32 result, not fp64 passed through
    # zero row: finite (ln_eps keeps the root away from zero), and zero out
    z = O.rmsnorm(np.zeros((1, 8), np.float32), np.ones(8, np.float32), 1e-6)
    assert np.array_equal(z, np.zeros((1, 8), np.float32))
    # constant row: |c| / sqrt(c^2) = 1, sign kept
    c = O.rmsnorm(np.full((1, 16), -3.0, np.float32), np.ones(16, np.float32), 0.0)
    assert np.allclose(c, -1.0, rtol=0, atol=1e-7)


def test_rotating_weights_and_activations_cancels():
    """The ablation's weight-and-activation variant multiplies W H by H x: H H = I, so without the
    quantisers the product is W x again.  Pins that the transform is its own inverse *as a matrix*
    applied on the feature axis of both operands (a transform along the wrong axis fails)."""
    rng = np.random.default_rng(11)
    K = 256
    W = rng.standard_normal((24, K)).astype(np.float32)
    x = rng.standard_normal((5, K)).astype(np.float32)
    got = O.fwht_rows(x).astype(np.float64) @ O.fwht_rows(W).astype(np.float64).T
    want = x.astype(np.float64) @ W.astype(np.float64).T
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()


# --- Low-bit Q/K/V head states (Section 3.1) ----------------------------------------------------------

def test_kv_absmax_hand_row(golden):
    c = golden["kv_absmax_hand_row"]
    x = np.array([c["x"]], np.float32)
    for bits in (4, 3):
        codes, packed, scales = O.kv_quant_absmax(x, bits, c["eps"][0])
        assert codes[0].tolist() == [int(v) for v in c[f"codes{bits}"]]
        assert packed[0].tolist() == [int(v) for v in c[f"packed{bits}"]]
        assert scales[0] == np.float32(c[f"scale{bits}"][0])


def test_kv_absmax_ties_go_to_even(golden):
    c = golden["kv_absmax_ties"]
    for bits in (4, 3):
        x = np.array([c[f"x{bits}"]], np.float32)
        codes, _, scales = O.kv_quant_absmax(x, bits, c["eps"][0])
        assert codes[0].tolist() == [int(v) for v in c[f"codes{bits}"]]
        assert scales[0] == 1.0


def test_kv_absmax_is_eq5_plus_128_at_8_bits():
    """At 8 bits the head-state quantiser must be the (separately pinned) INT8 absmax quantiser of Eq. 5 with an
    offset of 128, row for row, for both input types."""
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((37, 128)) * np.exp(rng.standard_normal((37, 1)))).astype(np.float32)
    x[3] = 0.0                                               # a zero row: codes 128, scale 0
    for xx in (x, synth.f32_to_bf16_bits(x)):
        q, s = O.fwht_quant(xx, 8, hadamard=False, eps=1e-5)
        codes, packed, scales = O.kv_quant_absmax(xx, 8, 1e-5)
        assert np.array_equal(codes.astype(np.int32) - 128, q.astype(np.int32))
        assert np.array_equal(packed, codes) and np.array_equal(scales, s)
    assert np.all(codes[3] == 128) and scales[3] == 0.0


@pytest.mark.parametrize("bits", [8, 4, 3])
def test_kv_absmax_invariants(bits):
    rng = np.random.default_rng(bits)
    rows, d = 64, 128
    x = (rng.standard_normal((rows, d)) * 3.0).astype(np.float32)
    x[:, 5] *= 20.0                                          # an outlier channel, as in K states
    half, qmax = 1 << (bits - 1), (1 << (bits - 1)) - 1
    codes, packed, scales = O.kv_quant_absmax(x, bits, 1e-5)
    assert codes.min() >= 0 and codes.max() <= 2 * half - 1
    # the row maximum maps to +-qmax exactly, and -2^(b-1) is never produced (|qmax h/(gamma+eps)| <= qmax)
    amax = np.abs(x).argmax(1)
    top = codes[np.arange(rows), amax].astype(np.int32) - half
    assert np.array_equal(top, np.sign(x[np.arange(rows), amax]).astype(np.int32) * qmax)
    assert codes.min() >= 1
    # reconstruction: within half a step of the scale (plus the eps shrink and fp32 rounding)
    xhat = O.kv_dequant(codes, scales, bits)
    assert np.all(np.abs(xhat - x) <= scales[:, None] * (0.5 + 1e-3))
    assert np.allclose(scales, np.abs(x).max(1) / qmax, rtol=1e-6)
    # scaling a row by a power of two scales the scale and leaves the codes alone (eps = 0)
    c1, _, s1 = O.kv_quant_absmax(x, bits, 0.0)
    c2, _, s2 = O.kv_quant_absmax(x * 4.0, bits, 0.0)
    assert np.array_equal(c1, c2) and np.array_equal(s2, s1 * 4.0)
    # the packed stream, unpacked bit by bit here
    bitsarr = np.unpackbits(packed, axis=1, bitorder="little").reshape(rows, d, bits)
    back = (bitsarr * (1 << np.arange(bits))).sum(2)
    assert np.array_equal(back, codes)
    # bf16 output of the inverse map: the fp32 result rounded to nearest even
    assert np.array_equal(O.kv_dequant(codes, scales, bits, out_bf16=True), synth.f32_to_bf16_bits(xhat))
