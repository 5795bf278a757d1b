"""Pins for the oracle's transform (Eq. 1-2) and sign generator.

None of these re-types the oracle's matrix formula: they compare against
brute-force complex DFT sums written here, against numpy's rfft, against closed
forms, and against the invariants the paper states (orthonormality, the
inverse being "unpack, irfft, apply s").
"""
import cmath
import math

import numpy as np
import pytest

from oracle import srft_oracle as O

TINY_D = [2, 4, 6, 8, 12, 16, 24, 32, 96]
ALL_D = TINY_D + [64, 128, 256]


def brute_force_pack(u):
    """pack(F u) by the definition: unitary DFT sums in complex arithmetic, then Eq. 2 by cases."""
    d = len(u)
    h = d // 2
    Y = []
    for k in range(h + 1):
        acc = 0j
        for n in range(d):
            acc += u[n] * cmath.exp(-2j * math.pi * k * n / d)
        Y.append(acc / math.sqrt(d))
    z = [0.0] * d
    for k in range(d):
        if k == 0:
            z[k] = Y[0].real
        elif k == h:
            z[k] = Y[h].real
        elif k < h:
            z[k] = math.sqrt(2) * Y[k].real
        else:
            z[k] = math.sqrt(2) * Y[k - h].imag
    return np.array(z)


@pytest.mark.parametrize("d", TINY_D)
def test_dense_and_fft_forms_equal_brute_force(d):
    rng = np.random.RandomState(d)
    x = rng.standard_normal(d)
    s = O.signs_from_seed(77 + d, d)
    ref = brute_force_pack(x * s)
    zd = O.srft_forward(x[None], s, form="dense")[0]
    zf = O.srft_forward(x[None], s, form="fft")[0]
    assert np.max(np.abs(zd - ref)) < 1e-12
    assert np.max(np.abs(zf - ref)) < 1e-12


@pytest.mark.parametrize("d", ALL_D)
def test_forms_equal_numpy_rfft(d):
    rng = np.random.RandomState(1000 + d)
    x = rng.standard_normal((5, d))
    s = O.signs_from_seed(d, d)
    Y = np.fft.rfft(x * s, norm="ortho", axis=-1)
    h = d // 2
    ref = np.empty((5, d))
    ref[:, 0] = Y[:, 0].real
    ref[:, h] = Y[:, h].real
    for k in range(1, h):
        ref[:, k] = math.sqrt(2) * Y[:, k].real
        ref[:, h + k] = math.sqrt(2) * Y[:, k].imag
    for form in ("dense", "fft"):
        z = O.srft_forward(x, s, form=form)
        assert np.max(np.abs(z - ref)) < 1e-12, form


@pytest.mark.parametrize("d", [8, 96, 128])
def test_mixed_radix_fft_equals_numpy_fft(d):
    rng = np.random.RandomState(5)
    a = rng.standard_normal((3, d)) + 1j * rng.standard_normal((3, d))
    assert np.max(np.abs(O.fft_mixed_radix(a) - np.fft.fft(a, axis=-1))) < 1e-11
    # lengths with other prime factors and a prime length
    for n in (15, 21, 7, 45):
        b = rng.standard_normal(n) + 1j * rng.standard_normal(n)
        assert np.max(np.abs(O.fft_mixed_radix(b) - np.fft.fft(b))) < 1e-11


@pytest.mark.parametrize("d", [8, 96, 128, 256])
def test_closed_forms(d):
    h = d // 2
    ones = np.ones(d, dtype=np.int8)
    n = np.arange(d)
    for form in ("dense", "fft"):
        # constant c -> only z_0 = c sqrt(d)
        z = O.srft_forward(np.full((1, d), 3.0), ones, form=form)[0]
        exp = np.zeros(d); exp[0] = 3.0 * math.sqrt(d)
        assert np.max(np.abs(z - exp)) < 1e-11
        # (-1)^n -> only z_{d/2} = sqrt(d)
        z = O.srft_forward(((-1.0) ** n)[None], ones, form=form)[0]
        exp = np.zeros(d); exp[h] = math.sqrt(d)
        assert np.max(np.abs(z - exp)) < 1e-11
        # unit impulse at n=0 -> Y_k = 1/sqrt(d) for all k: z_0 = z_h = 1/sqrt d, Re rows sqrt(2/d), Im rows 0
        e0 = np.zeros((1, d)); e0[0, 0] = 1.0
        z = O.srft_forward(e0, ones, form=form)[0]
        exp = np.zeros(d); exp[0] = exp[h] = 1 / math.sqrt(d); exp[1:h] = math.sqrt(2.0 / d)
        assert np.max(np.abs(z - exp)) < 1e-12
        # impulse at n=1 -> Y_k = exp(-2 pi i k/d)/sqrt d : Im rows are NEGATIVE sines (rfft sign convention)
        e1 = np.zeros((1, d)); e1[0, 1] = 1.0
        z = O.srft_forward(e1, ones, form=form)[0]
        for k in range(1, h):
            assert abs(z[k] - math.sqrt(2.0 / d) * math.cos(2 * math.pi * k / d)) < 1e-12
            assert abs(z[h + k] + math.sqrt(2.0 / d) * math.sin(2 * math.pi * k / d)) < 1e-12
        assert abs(z[h] + 1 / math.sqrt(d)) < 1e-12
        # cos(2 pi m n/d) -> only z_m = sqrt(d/2); sin(2 pi m n/d) -> only z_{h+m} = -sqrt(d/2)
        m = 3 if h > 3 else 1
        z = O.srft_forward(np.cos(2 * np.pi * m * n / d)[None], ones, form=form)[0]
        exp = np.zeros(d); exp[m] = math.sqrt(d / 2)
        assert np.max(np.abs(z - exp)) < 1e-11
        z = O.srft_forward(np.sin(2 * np.pi * m * n / d)[None], ones, form=form)[0]
        exp = np.zeros(d); exp[h + m] = -math.sqrt(d / 2)
        assert np.max(np.abs(z - exp)) < 1e-11


@pytest.mark.parametrize("d", [6, 32, 96, 128, 256])
def test_sign_diagonal_is_applied_to_the_input_side(d):
    # SRFT = pack(F diag(s) x): flipping s_n negates the contribution of x_n only.
    rng = np.random.RandomState(3)
    x = rng.standard_normal((1, d))
    s = np.ones(d, dtype=np.int8)
    z0 = O.srft_forward(x, s)
    s2 = s.copy(); s2[5 % d] = -1
    x2 = x.copy(); x2[0, 5 % d] *= -1
    assert np.allclose(O.srft_forward(x, s2), O.srft_forward(x2, s), atol=1e-13)
    assert not np.allclose(O.srft_forward(x, s2), z0)


@pytest.mark.parametrize("d", ALL_D)
def test_orthonormal(d):
    Q = O.srft_matrix(d)
    assert np.max(np.abs(Q @ Q.T - np.eye(d))) < 1e-12
    assert np.max(np.abs(Q.T @ Q - np.eye(d))) < 1e-12
    rng = np.random.RandomState(d)
    x = rng.standard_normal((4, d)); y = rng.standard_normal((4, d))
    s = O.signs_from_seed(9, d)
    for form in ("dense", "fft"):
        zx, zy = O.srft_forward(x, s, form=form), O.srft_forward(y, s, form=form)
        assert np.allclose(np.linalg.norm(zx, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)
        assert np.allclose((zx * zy).sum(1), (x * y).sum(1), atol=1e-11)


@pytest.mark.parametrize("d", ALL_D)
def test_inverse_round_trip_double(d):
    rng = np.random.RandomState(d + 1)
    x = rng.standard_normal((6, d))
    s = O.signs_from_seed(31, d)
    for f1 in ("dense", "fft"):
        for f2 in ("dense", "fft"):
            back = O.srft_inverse(O.srft_forward(x, s, form=f1), s, form=f2)
            assert np.max(np.abs(back - x)) < 1e-12, (f1, f2)


@pytest.mark.parametrize("d", [64, 96, 128, 256])
def test_inverse_is_unpack_irfft_sign(d):
    # the sentence after Eq. 2, with numpy's irfft as the library witness
    rng = np.random.RandomState(2 * d)
    z = rng.standard_normal((3, d))
    s = O.signs_from_seed(5, d)
    h = d // 2
    Y = np.zeros((3, h + 1), dtype=complex)
    Y[:, 0] = z[:, 0]; Y[:, h] = z[:, h]
    Y[:, 1:h] = (z[:, 1:h] + 1j * z[:, h + 1:]) / math.sqrt(2)
    ref = np.fft.irfft(Y, n=d, norm="ortho", axis=-1) * s
    for form in ("dense", "fft"):
        assert np.max(np.abs(O.srft_inverse(z, s, form=form) - ref)) < 1e-12


@pytest.mark.parametrize("d", [64, 96, 128, 256])
def test_fp32_round_trip_without_quantization(d):
    # norms preserved and x recovered within 1e-5 relative error in fp32 (paper: ~1e-6)
    rng = np.random.RandomState(d)
    x = rng.standard_normal((64, d)).astype(np.float16)
    s = O.signs_from_seed(123, d)
    z = O.srft_forward(x, s, dtype=np.float32)
    assert z.dtype == np.float32
    back = O.srft_inverse(z, s, dtype=np.float32)
    xf = x.astype(np.float64)
    rel = np.linalg.norm(back - xf, axis=1) / np.linalg.norm(xf, axis=1)
    assert rel.max() < 1e-5
    nrm = np.abs(np.linalg.norm(z.astype(np.float64), axis=1) / np.linalg.norm(xf, axis=1) - 1)
    assert nrm.max() < 1e-5


def test_gaussianization_of_an_outlier_channel():
    # Sec. 3.1: a heavy-tailed input becomes near-Gaussian after SRFT (qualitative pin).
    d = 128
    rng = np.random.RandomState(0)
    x = rng.standard_normal((2000, d)); x[:, 17] *= 30.0

    def excess_kurtosis(v):
        v = v - v.mean()
        return (v ** 4).mean() / (v ** 2).mean() ** 2 - 3.0

    s = O.signs_from_seed(1, d)
    z = O.srft_forward(x, s)
    assert excess_kurtosis(x.ravel()) > 50
    assert abs(excess_kurtosis(z.ravel())) < 3.0   # scale mixture over k of the outlier's cos/sin weights
    # energy is spread: no packed coordinate holds more than a few percent
    frac = (z ** 2).mean(0) / (z ** 2).mean(0).sum()
    assert frac.max() < 0.05


def test_splitmix64_reference_values():
    # first outputs of the published splitmix64 for seed 1234567 (widely used test vector)
    assert O.splitmix64_stream(1234567, 5) == [
        6457827717110365317, 3203168211198807973, 9817491932198370423,
        4593380528125082431, 16408922859458223821]


def test_signs_are_pm1_and_balanced():
    s = O.signs_from_seed(42, 4096)
    assert s.dtype == np.int8 and set(np.unique(s)) == {-1, 1}
    assert abs(int(s.sum())) < 4 * 64          # 4 sigma for 4096 fair coins
    assert np.array_equal(s[:128], O.signs_from_seed(42, 128))   # prefix property
    assert not np.array_equal(O.signs_from_seed(43, 128), s[:128])
    v = O.splitmix64_stream(42, 8)
    assert [(-1 if x >> 63 else 1) for x in v] == list(s[:8])


# ----------------------------------------------------------------------------- the SRHT comparator
def test_hadamard_matrix_against_scipy_the_entry_formula_and_a_butterfly():
    import scipy.linalg
    for d in (1, 2, 4, 32, 64, 128, 256):
        H = O.hadamard_matrix(d)
        assert np.allclose(H, scipy.linalg.hadamard(d) / np.sqrt(d), atol=1e-15)
        assert np.allclose(H @ H.T, np.eye(d), atol=1e-12) and np.array_equal(H, H.T)
    d = 64
    H = O.hadamard_matrix(d)
    p, n = np.meshgrid(np.arange(d), np.arange(d), indexing="ij")
    parity = np.array([[bin(a & b).count("1") & 1 for b in range(d)] for a in range(d)])
    assert np.allclose(H * np.sqrt(d), 1 - 2 * parity)                    # (-1)^popcount(p & n)
    # in-place butterflies (the fast Walsh-Hadamard transform) give the same product
    rng = np.random.RandomState(0)
    u = rng.standard_normal(d)
    a = u.copy()
    h = 1
    while h < d:
        for i in range(0, d, 2 * h):
            for j in range(i, i + h):
                a[j], a[j + h] = a[j] + a[j + h], a[j] - a[j + h]
        h *= 2
    assert np.allclose(a / np.sqrt(d), H @ u, atol=1e-12)
    with pytest.raises(ValueError):
        O.hadamard_matrix(96)


def test_srht_form_round_trips_and_keeps_norms():
    d = 128
    rng = np.random.RandomState(1)
    x = rng.standard_normal((20, d))
    s = O.signs_from_seed(3, d)
    z = O.srft_forward(x, s, form="hadamard")
    assert np.allclose(np.linalg.norm(z, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)
    assert np.allclose(O.srft_inverse(z, s, form="hadamard"), x, atol=1e-12)
    # s * ones -> all energy in coefficient 0
    z1 = O.srft_forward((s * 2.0)[None, :], s, form="hadamard")
    assert abs(z1[0, 0] - 2.0 * np.sqrt(d)) < 1e-12 and np.all(np.abs(z1[0, 1:]) < 1e-12)


def test_srft_and_srht_gaussianize_alike():
    """Sec. 3.1: heavy-tailed channels give large excess kurtosis; after either transform the coefficients are
    near-Gaussian (the paper reports about -0.5 after SRFT, "matching SRHT's behavior"), and the 4-bit
    reconstruction errors agree (Sec. 1: "statistically indistinguishable").  Synthetic stand-in for the paper's
    activations: N(0,1) times per-channel gains ~ lognormal(0, 1)."""
    d, n = 128, 4000
    rng = np.random.RandomState(2)
    x = (rng.standard_normal((n, d)) * np.exp(rng.standard_normal(d))).astype(np.float16)
    s = O.signs_from_seed(5, d)

    def excess_kurtosis(v):
        v = v - v.mean(axis=1, keepdims=True)
        return ((v ** 4).mean(axis=1) / (v ** 2).mean(axis=1) ** 2 - 3.0).mean()

    assert excess_kurtosis(x.astype(np.float64)) > 10
    lam = np.ones(d, dtype=np.float32)
    mse, kurt = {}, {}
    for form in ("dense", "hadamard"):
        kurt[form] = excess_kurtosis(O.srft_forward(x, s, form=form))
        q = O.quantize(x, s, lam, 32, form=form)
        back = O.dequantize_f64(q["codes"], q["scales"], s, lam, 32, form=form)
        mse[form] = np.mean((back - x.astype(np.float64)) ** 2)
    assert -1.0 < kurt["dense"] < 0.5 and -1.0 < kurt["hadamard"] < 0.5
    assert abs(mse["dense"] - mse["hadamard"]) / mse["dense"] < 0.1
    # and both beat quantizing the raw vectors (identity in place of the transform would keep the loud channels)
    g = 32
    xr = x.astype(np.float64).reshape(n, d // g, g)
    sc = np.abs(xr).max(axis=-1, keepdims=True) / 7
    raw_mse = np.mean((np.rint(xr / sc) * sc - xr) ** 2)
    assert mse["dense"] < raw_mse and mse["hadamard"] < raw_mse


@pytest.mark.parametrize("d", [96, 128, 256])
def test_inverse_transform_folds_twice_over_cosine_sine_and_code_parity(d):
    """The symmetries of Q (Eq. 1-2) that the read kernels at d = 128 and 256 rest on, checked on the oracle's matrix.

    With h = d/2, C the part of Q^T z from the packed indices p <= h (DC, cosine rows, Nyquist) and S the part from
    p > h (sine rows): C_{d-n} = C_n, S_{d-n} = -S_n; and under n -> h - n an even p keeps (cosine) or flips (sine) its
    sign, an odd p the other way round.  So with Ce, Co, Se, So the sums over even / odd p, the four outputs m, d - m,
    h - m, h + m follow from four numbers, for m = 0 .. d/4; Co and Se vanish at m = d/4, So and Se at m = 0.
    """
    rng = np.random.RandomState(d)
    h = d // 2
    Q = O.srft_matrix(d)
    z = rng.standard_normal(d)
    u = Q.T @ z
    p = np.arange(d)
    cos_side, sin_side = p <= h, p > h
    even, odd = p % 2 == 0, p % 2 == 1

    def part(mask, n):
        return Q[mask, n] @ z[mask]

    for m in range(d // 4 + 1):
        ce, co = part(cos_side & even, m), part(cos_side & odd, m)
        se, so = part(sin_side & even, m), part(sin_side & odd, m)
        assert abs(u[m] - (ce + co + so + se)) < 1e-12
        assert abs(u[(d - m) % d] - (ce + co - so - se)) < 1e-12
        assert abs(u[h - m] - (ce - co + so - se)) < 1e-12
        assert abs(u[(h + m) % d] - (ce - co - so + se)) < 1e-12
        if m == 0:
            assert abs(so) < 1e-12 and abs(se) < 1e-12
        if m == d // 4:
            assert abs(co) < 1e-12 and abs(se) < 1e-12
