"""Pins of the fp64 oracle against what the paper and the mathematics fix.

Nothing here touches the GPU library.  Every check compares the oracle with
something other than itself: a closed form, an invariant, a library routine
used on a special case, a brute force on tiny inputs, or a hand-built fixture.
"""
import math
import os

import numpy as np
import pytest
import scipy.integrate
import scipy.special
import scipy.stats

import oracle
from paper_2502_02617_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def S():
    return oracle.preconditioner(0)


@pytest.fixture(scope="module")
def cb():
    return oracle.default_codebooks()


@pytest.fixture(scope="module")
def X0():
    # config 0: 1024 vectors, d=128, fp32 N(0,1), seed 0
    return synth.gaussian_vectors(1024, seed=0).numpy().astype(np.float64)


# ----------------------------------------------------------------------------
# Preconditioner (Section 3.2 footnote: P^T P = I)
# ----------------------------------------------------------------------------
def test_S_is_orthogonal(S):
    assert np.linalg.norm(S.T @ S - np.eye(128)) <= 1e-12
    assert np.linalg.norm(S @ S.T - np.eye(128)) <= 1e-12
    assert abs(abs(np.linalg.det(S)) - 1.0) <= 1e-10


def test_S_matches_lapack_qr():
    # QR with positive diagonal of R is unique: LAPACK's factor, sign-fixed, must agree.
    G = oracle.gaussian_matrix(5)
    S = oracle.rotation_from_gaussian(G)
    Q, R = np.linalg.qr(G)
    Qs = Q * np.sign(np.diag(R))[None, :]
    assert np.max(np.abs(S - Qs)) <= 1e-11
    # S^T G is upper triangular with positive diagonal
    Rm = S.T @ G
    assert np.max(np.abs(np.tril(Rm, -1))) <= 1e-11
    assert np.all(np.diag(Rm) > 0)


def test_S_preserves_inner_products(S):
    rng = np.random.default_rng(1)
    a, b = rng.standard_normal((2, 128))
    assert abs((a @ S) @ (b @ S) - a @ b) <= 1e-12 * 128
    assert abs(np.linalg.norm(a @ S) - np.linalg.norm(a)) <= 1e-12


def test_gaussian_matrix_is_standard_normal():
    G = oracle.gaussian_matrix(0)
    assert G.shape == (128, 128)
    # KS against N(0,1): 16384 samples
    d, p = scipy.stats.kstest(G.ravel(), "norm")
    assert p > 1e-3, (d, p)
    assert not np.array_equal(G, oracle.gaussian_matrix(1))
    assert np.array_equal(G, oracle.gaussian_matrix(0))


# ----------------------------------------------------------------------------
# Polar transform (Definition 1, Algorithm 1 procedure Polar)
# ----------------------------------------------------------------------------
def test_polar_d2_is_textbook():
    for a, b in [(3.0, 4.0), (-1.0, 2.0), (-2.0, -0.5), (0.7, -0.1), (1.0, 0.0), (0.0, 0.0)]:
        psi, r = oracle.polar([a, b], 1)
        assert abs(r[0] - math.hypot(a, b)) <= 1e-15
        ref = math.atan2(b, a) % (2 * math.pi)
        assert abs(psi[0] - ref) <= 1e-15
        assert 0.0 <= psi[0] < 2 * math.pi + 1e-15


def test_polar_round_trip_exact(S, X0):
    # quantisation disabled: x -> xS -> Polar -> inverse -> S^T
    Y = X0[:64] @ S
    for y in Y:
        psi, r = oracle.polar(y, 4)
        assert psi.size == 120 and r.size == 8
        y2 = oracle.polar_inverse(psi, r, 128, 4)
        assert np.max(np.abs(y2 - y)) <= 1e-12
        x2 = y2 @ S.T
        assert np.max(np.abs(x2 - y @ S.T)) <= 1e-12
    # full depth too (Definition 1: log2 d levels, one radius)
    psi, r = oracle.polar(Y[0], 7)
    assert psi.size == 127 and r.size == 1
    assert abs(r[0] - np.linalg.norm(Y[0])) <= 1e-12
    assert np.max(np.abs(oracle.polar_inverse(psi, r, 128, 7) - Y[0])) <= 1e-12


def test_final_radius_is_block_norm(S, X0):
    Y = X0[:64] @ S
    for y in Y:
        _, r = oracle.polar(y, 4)
        ref = np.linalg.norm(y.reshape(8, 16), axis=1)
        assert np.max(np.abs(r - ref)) <= 1e-12


def test_angle_ranges_and_definition(S, X0):
    y = (X0[:1] @ S)[0]
    psi, _ = oracle.polar(y, 4)
    l1, l2, l3, l4 = psi[:64], psi[64:96], psi[96:112], psi[112:120]
    assert np.all((l1 >= 0) & (l1 < 2 * np.pi))
    for lv in (l2, l3, l4):
        assert np.all((lv >= 0) & (lv <= np.pi / 2))
    # Definition 1, level l >= 2: tan psi = norm of the upper half / norm of the lower half
    for lev, ang in ((2, l2), (3, l3), (4, l4)):
        w = 2 ** lev
        seg = y.reshape(-1, w)
        lo = np.linalg.norm(seg[:, : w // 2], axis=1)
        hi = np.linalg.norm(seg[:, w // 2 :], axis=1)
        assert np.max(np.abs(np.arctan2(hi, lo) - ang)) <= 1e-13
    assert np.max(np.abs(np.mod(np.arctan2(y[1::2], y[0::2]), 2 * np.pi) - l1)) <= 1e-13


def test_inverse_matches_closed_product_form(S, X0):
    # Definition 1's reverse map, 0-based: x_i = r * prod_l (cos if (i mod 2^l) < 2^(l-1) else sin)(psi^(l)_{i >> l})
    y = (X0[3:4] @ S)[0]
    psi, r = oracle.polar(y, 4)
    off = {1: 0, 2: 64, 3: 96, 4: 112}
    for i in range(128):
        v = r[i >> 4]
        for l in range(1, 5):
            a = psi[off[l] + (i >> l)]
            v *= math.cos(a) if (i % (1 << l)) < (1 << (l - 1)) else math.sin(a)
        assert abs(v - y[i]) <= 1e-12


# ----------------------------------------------------------------------------
# Angle densities (Lemma 2)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("level", [2, 3, 4, 5])
def test_pdf_normalised_symmetric(level):
    f = lambda t: oracle.angle_pdf(level, t)
    total, _ = scipy.integrate.quad(f, 0, np.pi / 2, epsabs=1e-13, epsrel=1e-13)
    assert abs(total - 1.0) <= 1e-11
    for t in (0.1, 0.3, 0.7):
        assert abs(f(t) - f(np.pi / 2 - t)) <= 1e-13
    mean, _ = scipy.integrate.quad(lambda t: t * f(t), 0, np.pi / 2, epsabs=1e-13, epsrel=1e-13)
    assert abs(mean - np.pi / 4) <= 1e-11
    # the printed constant: Gamma(2^(l-1)) / (2^(2^(l-1)-2) Gamma(2^(l-2))^2) at psi = pi/4
    n = 2 ** (level - 1)
    const = math.gamma(n) / (2 ** (n - 2) * math.gamma(n / 2) ** 2)
    assert abs(f(np.pi / 4) - const) <= 1e-12 * const


def test_empirical_angles_follow_lemma2(S, X0):
    # Gaussian vectors, rotated: level 1 uniform on [0, 2pi); level l >= 2 has
    # sin^2(psi) ~ Beta(2^(l-2), 2^(l-2)), i.e. CDF = regularised incomplete beta.
    Y = X0 @ S
    psi = np.stack([oracle.polar(y, 4)[0] for y in Y])
    lv = {1: psi[:, :64].ravel(), 2: psi[:, 64:96].ravel(), 3: psi[:, 96:112].ravel(), 4: psi[:, 112:].ravel()}
    assert lv[1].size == 65536 and lv[4].size == 8192
    d, p = scipy.stats.kstest(lv[1], lambda t: t / (2 * np.pi))
    assert p > 1e-3, ("level 1", d, p)
    for l in (2, 3, 4):
        a = 2.0 ** (l - 2)
        d, p = scipy.stats.kstest(lv[l], lambda t: scipy.special.betainc(a, a, np.sin(t) ** 2))
        assert p > 1e-3, (l, d, p)
    # the oracle's pdf integrates to that same CDF
    for l in (2, 3, 4):
        a = 2.0 ** (l - 2)
        for t in (0.4, 0.9, 1.3):
            F, _ = scipy.integrate.quad(lambda u: oracle.angle_pdf(l, u), 0, t, epsabs=1e-13)
            assert abs(F - scipy.special.betainc(a, a, math.sin(t) ** 2)) <= 1e-10


# ----------------------------------------------------------------------------
# Codebooks (Eq. 3)
# ----------------------------------------------------------------------------
def test_level1_codebook_closed_form():
    c, b = oracle.codebook(1, 16)
    assert np.max(np.abs(c - (np.arange(16) + 0.5) * np.pi / 8)) <= 1e-15
    assert np.max(np.abs(b - np.arange(17) * np.pi / 8)) <= 1e-15
    # distortion of a uniform density on bins of width pi/8
    assert abs(oracle.codebook_distortion(1, c) - (np.pi / 8) ** 2 / 12) <= 1e-12


@pytest.mark.parametrize("level", [2, 3, 4])
def test_lloyd_max_fixed_point(level):
    c, b = oracle.codebook(level, 4)
    assert b[0] == 0.0 and abs(b[4] - np.pi / 2) <= 1e-15
    # symmetry of the density about pi/4
    assert np.max(np.abs(c + c[::-1] - np.pi / 2)) <= 1e-12
    assert abs(b[2] - np.pi / 4) <= 1e-12
    # midpoint condition
    assert np.max(np.abs(b[1:4] - 0.5 * (c[:-1] + c[1:]))) <= 1e-14
    # centroid condition with an independent adaptive quadrature and the beta form of the density
    a = 2.0 ** (level - 2)
    m = 2 ** (level - 1) - 1
    pdf = lambda t: math.sin(2 * t) ** m
    for k in range(4):
        num, _ = scipy.integrate.quad(lambda t: t * pdf(t), b[k], b[k + 1], epsabs=1e-14, epsrel=1e-14)
        den, _ = scipy.integrate.quad(pdf, b[k], b[k + 1], epsabs=1e-14, epsrel=1e-14)
        assert abs(num / den - c[k]) <= 1e-11
    # bin probabilities from the closed-form CDF sum to one and are symmetric
    F = scipy.special.betainc(a, a, np.sin(b) ** 2)
    pr = np.diff(F)
    assert abs(pr.sum() - 1.0) <= 1e-12 and abs(pr[0] - pr[3]) <= 1e-11 and abs(pr[1] - pr[2]) <= 1e-11


@pytest.mark.parametrize("level", [2, 3, 4])
def test_codebook_is_a_local_minimum_of_eq3(level):
    c, _ = oracle.codebook(level, 4)
    base = oracle.codebook_distortion(level, c)
    # independent evaluation of Eq. 3 for the same centroids
    m = 2 ** (level - 1) - 1
    norm, _ = scipy.integrate.quad(lambda t: math.sin(2 * t) ** m, 0, np.pi / 2)
    edges = np.concatenate([[0.0], 0.5 * (c[:-1] + c[1:]), [np.pi / 2]])
    ref = sum(
        scipy.integrate.quad(lambda t, k=k: (t - c[k]) ** 2 * math.sin(2 * t) ** m / norm, edges[k], edges[k + 1], epsabs=1e-14)[0]
        for k in range(4)
    )
    assert abs(base - ref) <= 1e-11
    rng = np.random.default_rng(level)
    for _ in range(20):
        c2 = np.sort(c + 1e-3 * rng.standard_normal(4))
        assert oracle.codebook_distortion(level, c2) > base
    # and far better than a uniform grid on [0, pi/2]
    assert base < oracle.codebook_distortion(level, (np.arange(4) + 0.5) * np.pi / 8)


def test_codebook_regression_values():
    # values derived independently during the survey of the paper (Lloyd-Max of Lemma 2's densities)
    rows = np.loadtxt(os.path.join(GOLDEN, "codebook_lloyd_max.txt"))
    for row in rows:
        level = int(row[0])
        c, _ = oracle.codebook(level, 4)
        assert np.max(np.abs(c - row[1:5])) <= 2e-9
        assert abs(oracle.codebook_distortion(level, c) - row[5]) <= 2e-7


def test_sampled_kmeans_converges_to_codebook():
    # the paper's own recipe: 1-D k-means on sampled angles approaches the same centroids
    rng = np.random.default_rng(7)
    for level in (2, 3, 4):
        a = 2.0 ** (level - 2)
        t = np.arcsin(np.sqrt(rng.beta(a, a, size=400000)))
        c, _ = oracle.codebook(level, 4)
        km = (np.arange(4) + 0.5) * np.pi / 8
        for _ in range(200):
            edges = 0.5 * (km[:-1] + km[1:])
            idx = np.searchsorted(edges, t)
            km = np.array([t[idx == k].mean() for k in range(4)])
        assert np.max(np.abs(km - c)) <= 4e-3


# ----------------------------------------------------------------------------
# Quant (nearest centroid)
# ----------------------------------------------------------------------------
def test_quant_is_brute_force_nearest(cb):
    rng = np.random.default_rng(3)
    for level in (1, 2, 3, 4):
        K = oracle.CB_K[level]
        theta = cb[oracle.CB_OFF[level] : oracle.CB_OFF[level] + K]
        hi = 2 * np.pi if level == 1 else np.pi / 2
        for psi in np.concatenate([rng.uniform(0, hi, 500), [0.0, hi]]):
            assert oracle.quant(psi, theta) == int(np.argmin(np.abs(theta - psi)))
    # ties go to the lower index
    assert oracle.quant(1.0, np.array([0.5, 1.5])) == 0


def test_quant_equals_interval_lookup(cb):
    # Eq. 3's partition: the intervals between midpoints are the nearest-centroid cells
    for level in (1, 2, 3, 4):
        K = oracle.CB_K[level]
        theta, bnd = oracle.codebook(level, K)
        hi = 2 * np.pi if level == 1 else np.pi / 2
        grid = np.linspace(0, hi, 20001)[1:-1]
        grid = grid[np.min(np.abs(grid[:, None] - bnd[None, 1:-1]), axis=1) > 1e-9]
        ref = np.searchsorted(bnd[1:-1], grid)
        got = np.array([oracle.quant(t, theta) for t in grid])
        assert np.array_equal(ref, got)


def test_code_frequencies_match_bin_probabilities(S, cb, X0):
    rec = oracle.encode(X0, S, cb)
    J, _ = oracle.unpack(rec)
    spans = {1: (0, 64), 2: (64, 96), 3: (96, 112), 4: (112, 120)}
    for level, (a0, a1) in spans.items():
        K = oracle.CB_K[level]
        codes = J[:, a0:a1].ravel()
        n = codes.size
        freq = np.bincount(codes, minlength=K) / n
        if level == 1:
            prob = np.full(16, 1 / 16)
        else:
            _, bnd = oracle.codebook(level, 4)
            a = 2.0 ** (level - 2)
            prob = np.diff(scipy.special.betainc(a, a, np.sin(bnd) ** 2))
        sigma = np.sqrt(prob * (1 - prob) / n)
        assert np.all(np.abs(freq - prob) <= 4.5 * sigma), (level, freq, prob)


# ----------------------------------------------------------------------------
# binary16 conversion
# ----------------------------------------------------------------------------
def test_f16_conversion_matches_numpy():
    rng = np.random.default_rng(11)
    vals = np.concatenate([
        rng.standard_normal(2000) * 10.0 ** rng.uniform(-8, 5, 2000),
        [0.0, 1.0, 65504.0, 65519.9, 65520.0, 1e6, 2.0 ** -14, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -24,
         2.0 ** -25 * 1.0000001, 1.00048828125, 1.0009765625 + 2.0 ** -11, 1023.5 * 2.0 ** -24, -3.3],
    ])
    for v in vals:
        with np.errstate(over="ignore"):
            ref = int(np.float64(v).astype(np.float16).view(np.uint16))
        assert oracle.f64_to_f16(v) == ref, v
    for h in list(range(0, 0x7C00, 7)) + [0x7BFF, 0x0001, 0x03FF, 0x0400]:
        assert oracle.f16_to_f64(h) == float(np.uint16(h).view(np.float16))


# ----------------------------------------------------------------------------
# Record layout (Section 4.1: 46 code bits + 16 radius bits per 16 coordinates)
# ----------------------------------------------------------------------------
def test_record_size_and_bit_budget():
    assert oracle.REC == 62
    assert 62 * 8 / 128 == 3.875
    assert abs(16 * 128 / (62 * 8) - 4.129) < 1e-3


def test_pack_hand_built_record():
    # fixture written by hand from the documented canonical order
    lines = [l.split("#")[0].strip() for l in open(os.path.join(GOLDEN, "record_hand_built.txt"))]
    lines = [l for l in lines if l]
    codes = np.array([int(t) for t in lines[0].split()], dtype=np.int32)
    radii = np.array([int(t, 16) for t in lines[1].split()], dtype=np.uint16)
    expect = np.array([int(t, 16) for t in " ".join(lines[2:]).split()], dtype=np.uint8)
    assert codes.size == 120 and radii.size == 8 and expect.size == 62
    rec = oracle.pack(codes[None, :], radii[None, :])
    assert np.array_equal(rec[0], expect)
    J, r = oracle.unpack(rec)
    assert np.array_equal(J[0], codes) and np.array_equal(r[0], radii)


def test_pack_unpack_identity():
    rng = np.random.default_rng(5)
    J = np.concatenate([rng.integers(0, 16, (50, 64)), rng.integers(0, 4, (50, 56))], axis=1).astype(np.int32)
    rad = rng.integers(0, 0x7C00, (50, 8)).astype(np.uint16)
    rec = oracle.pack(J, rad)
    assert rec.shape == (50, 62)
    J2, rad2 = oracle.unpack(rec)
    assert np.array_equal(J, J2) and np.array_equal(rad, rad2)


# ----------------------------------------------------------------------------
# Encode / DeQuant
# ----------------------------------------------------------------------------
def test_encode_is_polar_plus_quant(S, cb, X0):
    rec, psi, Y = oracle.encode(X0[:32], S, cb, want_psi=True, want_y=True)
    assert np.max(np.abs(Y - X0[:32] @ S)) <= 1e-12
    J, rad = oracle.unpack(rec)
    for i in range(32):
        p, r = oracle.polar(Y[i], 4)
        assert np.max(np.abs(p - psi[i])) == 0.0
        spans = {1: (0, 64), 2: (64, 96), 3: (96, 112), 4: (112, 120)}
        for level, (a0, a1) in spans.items():
            theta = cb[oracle.CB_OFF[level] : oracle.CB_OFF[level] + oracle.CB_K[level]]
            ref = np.argmin(np.abs(theta[None, :] - p[a0:a1, None]), axis=1)
            assert np.array_equal(ref, J[i, a0:a1])
        assert np.array_equal(rad[i], r.astype(np.float16).view(np.uint16))


def test_dequant_block_lies_on_stored_sphere(S, cb, X0):
    rec = oracle.encode(X0[:64], S, cb)
    yhat = oracle.decode(rec, S, cb, rotated=True)
    _, rad = oracle.unpack(rec)
    r = rad.view(np.float16).astype(np.float64)
    assert np.max(np.abs(np.linalg.norm(yhat.reshape(64, 8, 16), axis=2) - r)) <= 1e-12
    xhat = oracle.decode(rec, S, cb, rotated=False)
    assert np.max(np.abs(xhat - yhat @ S.T)) <= 1e-12
    assert np.max(np.abs(np.linalg.norm(xhat, axis=1) - np.linalg.norm(r, axis=1))) <= 1e-12


def test_zero_vector_encodes_to_zero_radius(S, cb):
    rec = oracle.encode(np.zeros((1, 128)), S, cb)
    J, rad = oracle.unpack(rec)
    assert np.all(rad == 0) and np.all(J == 0)
    assert np.all(oracle.decode(rec, S, cb) == 0.0)


def test_reconstruction_error_matches_per_level_prediction(S, cb, X0):
    # For Gaussian data the angle errors of different levels are independent, so
    # E<x, xhat>/|x|^2 = prod_l E[cos(delta_l)] and |xhat| = |x| up to fp16:
    # relative L2 error = sqrt(2 (1 - prod_l E cos delta_l)).
    prod = 1.0
    for level in (1, 2, 3, 4):
        K = oracle.CB_K[level]
        c, b = oracle.codebook(level, K)
        m = 0 if level == 1 else 2 ** (level - 1) - 1
        pdf = lambda t: math.sin(2 * t) ** m if level > 1 else 1.0
        norm, _ = scipy.integrate.quad(pdf, b[0], b[-1])
        e = sum(
            scipy.integrate.quad(lambda t, k=k: math.cos(t - c[k]) * pdf(t), b[k], b[k + 1])[0] for k in range(K)
        ) / norm
        prod *= e
    predicted = math.sqrt(2 * (1 - prod))
    rec = oracle.encode(X0, S, cb)
    xhat = oracle.decode(rec, S, cb)
    rel = np.linalg.norm(xhat - X0) / np.linalg.norm(X0)
    assert abs(rel - predicted) <= 0.004, (rel, predicted)
    assert 0.17 < rel < 0.19


# ----------------------------------------------------------------------------
# Attention (Eq. 5)
# ----------------------------------------------------------------------------
def _small_cache(S, cb, T=37, Hkv=2, B=2, seed=21):
    k = synth.kv_stream(T * B, Hkv, seed).float().numpy().astype(np.float64)
    v = synth.kv_stream(T * B, Hkv, seed + 1).float().numpy().astype(np.float64)
    k_rec = oracle.encode(k.reshape(-1, 128), S, cb).reshape(Hkv, T * B, 62)
    v_rec = oracle.encode(v.reshape(-1, 128), S, cb).reshape(Hkv, T * B, 62)
    q = synth.queries(B, 4 * Hkv, seed).float().numpy().astype(np.float64)
    return q, k_rec, v_rec


def test_attention_is_textbook_softmax_on_dequantised_cache(S, cb):
    T, Hkv, B = 37, 2, 2
    q, k_rec, v_rec = _small_cache(S, cb, T, Hkv, B)
    seq_start = np.array([0, T], dtype=np.int64)
    ctx_len = np.array([T, T - 5], dtype=np.int32)
    scale = 1 / math.sqrt(128)
    out = oracle.attention(q, k_rec, v_rec, seq_start, ctx_len, S, cb, scale)
    for b in range(B):
        for h in range(4 * Hkv):
            hk = h // 4
            sl = slice(seq_start[b], seq_start[b] + ctx_len[b])
            Kh = oracle.decode(k_rec[hk, sl], S, cb)
            Vh = oracle.decode(v_rec[hk, sl], S, cb)
            p = scipy.special.softmax(Kh @ q[b, h] * scale)
            assert np.max(np.abs(p @ Vh - out[b, h])) <= 1e-12
    # rotated-domain evaluation (query rotated once, output un-rotated once) is the same number
    out_r = oracle.attention(q, k_rec, v_rec, seq_start, ctx_len, S, cb, scale, rotated=True)
    assert np.max(np.abs(out_r - out)) <= 1e-12


def test_attention_degenerate_cases(S, cb):
    T, Hkv, B = 9, 1, 2
    q, k_rec, v_rec = _small_cache(S, cb, T, Hkv, B, seed=33)
    scale = 1 / math.sqrt(128)
    # one cached token: the output is that token's dequantised value; empty context: zeros
    out = oracle.attention(q, k_rec, v_rec, np.array([3, 0]), np.array([1, 0], dtype=np.int32), S, cb, scale)
    assert np.max(np.abs(out[0] - oracle.decode(v_rec[0, 3:4], S, cb))) <= 1e-12
    assert np.all(out[1] == 0.0)
    # zero query: all scores equal, output = mean of the dequantised values
    out = oracle.attention(np.zeros_like(q), k_rec, v_rec, np.array([0, T]), np.array([T, T], dtype=np.int32), S, cb, scale)
    assert np.max(np.abs(out[0, 0] - oracle.decode(v_rec[0, :T], S, cb).mean(axis=0))) <= 1e-12


def test_hybrid_attention_is_one_softmax_over_prefix_and_window(S, cb):
    """Quantised prefix + unquantised window (Section 5.3's protocol): the textbook softmax over the
    concatenation of the dequantised prefix rows and the window rows, from scipy; an empty window reduces
    it to Eq. 5, an empty prefix to plain attention on the window, and it equals the log-sum-exp merge of
    the two separate attentions."""
    T, Hkv, B, cap = 29, 2, 3, 11
    q, k_rec, v_rec = _small_cache(S, cb, T, Hkv, B, seed=71)
    rng = np.random.default_rng(72)
    win_k = rng.standard_normal((B, Hkv, cap, 128))
    win_v = rng.standard_normal((B, Hkv, cap, 128))
    seq_start = np.array([0, T, 2 * T], dtype=np.int64)
    ctx_len = np.array([T, 0, T - 7], dtype=np.int32)
    win_len = np.array([cap, 5, 0], dtype=np.int32)
    scale = 1 / math.sqrt(128)
    out = oracle.attention_hybrid(q, k_rec, v_rec, seq_start, ctx_len, win_k, win_v, win_len, S, cb, scale)
    for b in range(B):
        for h in range(4 * Hkv):
            hk = h // 4
            sl = slice(seq_start[b], seq_start[b] + ctx_len[b])
            Kh = np.concatenate([oracle.decode(k_rec[hk, sl], S, cb).reshape(-1, 128), win_k[b, hk, :win_len[b]]])
            Vh = np.concatenate([oracle.decode(v_rec[hk, sl], S, cb).reshape(-1, 128), win_v[b, hk, :win_len[b]]])
            p = scipy.special.softmax(Kh @ q[b, h] * scale)
            assert np.max(np.abs(p @ Vh - out[b, h])) <= 1e-12
    # empty window: Eq. 5 on the cache alone
    plain = oracle.attention(q, k_rec, v_rec, seq_start, ctx_len, S, cb, scale)
    assert np.max(np.abs(out[2] - plain[2])) <= 1e-12
    # empty prefix: plain attention on the window rows
    for h in range(4 * Hkv):
        ref = oracle.attention_exact(q[1, h], win_k[1, h // 4, :5], win_v[1, h // 4, :5], scale)
        assert np.max(np.abs(out[1, h] - ref[0])) <= 1e-12
    # merge of the two separate results with their log-sum-exp weights
    for h in range(4 * Hkv):
        hk = h // 4
        Kp = oracle.decode(k_rec[hk, :T], S, cb)
        lse_p = scipy.special.logsumexp(Kp @ q[0, h] * scale)
        lse_w = scipy.special.logsumexp(win_k[0, hk] @ q[0, h] * scale)
        o_w = oracle.attention_exact(q[0, h], win_k[0, hk], win_v[0, hk], scale)[0]
        wp, ww = scipy.special.softmax([lse_p, lse_w])
        assert np.max(np.abs(wp * plain[0, h] + ww * o_w - out[0, h])) <= 1e-12
    # nothing at all: zeros
    none = oracle.attention_hybrid(q, k_rec, v_rec, seq_start, np.zeros(B, np.int32), win_k, win_v,
                                   np.zeros(B, np.int32), S, cb, scale)
    assert np.all(none == 0.0)


def test_online_codebook_fit_is_kmeans_on_the_angles(S, cb):
    """Section 4.1's online codebook: k-means on the sampled angles.  Against scikit-learn's Lloyd from the
    same start (its 1-D nearest-centroid rule is the same), the decrease of the sample distortion, the
    convergence towards the analytic codebook on Gaussian data (where the samples follow Lemma 2's
    densities), and zero iterations = the start."""
    from sklearn.cluster import KMeans

    x = synth.gaussian_vectors(3000, seed=81).numpy().astype(np.float64)
    _, psi, _ = oracle.encode(x, S, cb, want_psi=True, want_y=True)
    psi = psi.reshape(-1, 120)
    start = cb.copy()
    rng = np.random.default_rng(82)
    start[:16] += rng.uniform(-0.1, 0.1, 16)
    start[16:] += rng.uniform(-0.05, 0.05, 12)
    assert np.array_equal(oracle.fit_codebooks(x, S, start, 0), start)
    iters = 5
    fit = oracle.fit_codebooks(x, S, start, iters)
    cols = [(0, 64, 0, 16), (64, 96, 16, 20), (96, 112, 20, 24), (112, 120, 24, 28)]
    for a0, a1, c0, c1 in cols:
        samples = psi[:, a0:a1].reshape(-1, 1)
        km = KMeans(n_clusters=c1 - c0, init=start[c0:c1].reshape(-1, 1), n_init=1, max_iter=iters, tol=0.0,
                    algorithm="lloyd").fit(samples)
        assert np.max(np.abs(np.sort(km.cluster_centers_.ravel()) - fit[c0:c1])) <= 1e-9

        def distortion(c):
            return np.mean(np.min((samples - c[None, :]) ** 2, axis=1))
        assert distortion(fit[c0:c1]) <= distortion(start[c0:c1])
    # many rounds on Gaussian data: close to the analytic optimum (sampling noise; on the flat level-1
    # density Lloyd's iteration also converges slowly)
    far = oracle.fit_codebooks(x, S, start, 40)
    assert np.max(np.abs(far[:16] - cb[:16])) <= 0.04
    assert np.max(np.abs(far[16:] - cb[16:])) <= 0.02


@pytest.mark.parametrize("bits", [(2, 2, 2), (3, 1, 2)])
def test_online_fit_of_upper_level_codebooks(S, bits):
    """The same k-means for the angles of levels 5-7 (one vector gives 4, 2 and 1 of them): against
    scikit-learn's Lloyd from the same start, the decrease of the sample distortion, the approach to
    the Lloyd-Max quantisers of Lemma 2's densities on Gaussian data, and zero iterations = the start."""
    from sklearn.cluster import KMeans

    x = synth.gaussian_vectors(6000, seed=91).numpy().astype(np.float64)
    cbt = oracle.upper_codebooks(bits)
    _, psi, _ = oracle.encode_deep(x, S, oracle.default_codebooks(), bits, cbt, want_psi=True, want_y=True)
    psi = psi.reshape(-1, 127)
    start = cbt.copy()
    rng = np.random.default_rng(92)
    for l in range(3):
        start[l, : 1 << bits[l]] += rng.uniform(-0.02, 0.02, 1 << bits[l])
    assert np.array_equal(oracle.fit_upper_codebooks(x, S, bits, start, 0), start)
    iters = 5
    fit = oracle.fit_upper_codebooks(x, S, bits, start, iters)
    for l, (a0, a1) in enumerate(((120, 124), (124, 126), (126, 127))):
        K = 1 << bits[l]
        samples = psi[:, a0:a1].reshape(-1, 1)
        km = KMeans(n_clusters=K, init=start[l, :K].reshape(-1, 1), n_init=1, max_iter=iters, tol=0.0,
                    algorithm="lloyd").fit(samples)
        assert np.max(np.abs(np.sort(km.cluster_centers_.ravel()) - fit[l, :K])) <= 1e-9

        def distortion(c):
            return np.mean(np.min((samples - c[None, :]) ** 2, axis=1))
        assert distortion(fit[l, :K]) <= distortion(start[l, :K])
        assert np.all(fit[l, K:] == start[l, K:])        # unused entries pass through
    far = oracle.fit_upper_codebooks(x, S, bits, start, 60)
    for l in range(3):
        K = 1 << bits[l]
        assert np.max(np.abs(far[l, :K] - cbt[l, :K])) <= 0.01   # sampling noise of 24000 / 12000 / 6000 angles


def test_exact_attention_helper_is_plain_softmax():
    rng = np.random.default_rng(2)
    K, V = rng.standard_normal((2, 50, 128))
    q = rng.standard_normal((4, 128))
    out = oracle.attention_exact(q, K, V, 0.1)
    ref = scipy.special.softmax(q @ K.T * 0.1, axis=1) @ V
    assert np.max(np.abs(out - ref)) <= 1e-12


# ----------------------------------------------------------------------------
# Full-depth recursion (Definition 1 / Algorithm 1 at L = log2 d = 7; Section 4's
# memory count b_FPN + sum of code bits), per-level codebook sizes for levels 5..7
# ----------------------------------------------------------------------------
DEEP_BITS = [(2, 2, 2), (3, 1, 1), (1, 3, 2)]


@pytest.mark.parametrize("level,K", [(5, 2), (5, 4), (6, 4), (6, 8), (7, 2), (7, 4), (7, 8)])
def test_upper_level_codebooks_are_lloyd_max(level, K):
    c, b = oracle.codebook(level, K)
    assert b[0] == 0.0 and abs(b[K] - np.pi / 2) <= 1e-15
    assert np.max(np.abs(c + c[::-1] - np.pi / 2)) <= 1e-11          # density symmetric about pi/4
    assert np.max(np.abs(b[1:K] - 0.5 * (c[:-1] + c[1:]))) <= 1e-14   # midpoint condition
    m = 2 ** (level - 1) - 1
    logpdf = lambda t: m * math.log(max(math.sin(2 * t), 1e-300))
    peak = 0.0                                                        # sin(2t) <= 1: no overflow
    for k in range(K):                                                # centroid condition, independent quadrature
        num, _ = scipy.integrate.quad(lambda t: t * math.exp(logpdf(t) - peak), b[k], b[k + 1], epsabs=0, epsrel=1e-13, limit=200)
        den, _ = scipy.integrate.quad(lambda t: math.exp(logpdf(t) - peak), b[k], b[k + 1], epsabs=0, epsrel=1e-13, limit=200)
        assert abs(num / den - c[k]) <= 1e-9, (k, num / den, c[k])
    # bin probabilities from the closed-form CDF (sin^2 psi ~ Beta(2^(l-2), 2^(l-2))) sum to one
    a = 2.0 ** (level - 2)
    pr = np.diff(scipy.special.betainc(a, a, np.sin(b) ** 2))
    assert abs(pr.sum() - 1.0) <= 1e-12 and np.max(np.abs(pr - pr[::-1])) <= 1e-10
    # the angle concentrates around pi/4 as the level rises (Lemma 1: variance O(1/d))
    assert oracle.codebook_distortion(level, c) < oracle.codebook_distortion(level - 1, oracle.codebook(level - 1, K)[0])


def test_upper_level_angles_follow_lemma2(S):
    Y = synth.gaussian_vectors(4096, seed=5).numpy().astype(np.float64) @ S
    psi = np.stack([oracle.polar(y, 7)[0] for y in Y])
    spans = {5: (120, 124), 6: (124, 126), 7: (126, 127)}
    for l, (a0, a1) in spans.items():
        a = 2.0 ** (l - 2)
        d, p = scipy.stats.kstest(psi[:, a0:a1].ravel(), lambda t: scipy.special.betainc(a, a, np.sin(t) ** 2))
        assert p > 1e-3, (l, d, p)
    # the first 120 angles are those of the depth-4 transform; the level-5 angles are built on its block radii
    p4, r4 = oracle.polar(Y[0], 4)
    assert np.array_equal(psi[0, :120], p4)
    assert np.max(np.abs(psi[0, 120:124] - np.arctan2(r4[1::2], r4[0::2]))) <= 1e-15


@pytest.mark.parametrize("bits", DEEP_BITS)
def test_deep_record_structure(S, cb, X0, bits):
    cbt = oracle.upper_codebooks(bits)
    rec, psi, Y = oracle.encode_deep(X0[:200], S, cb, bits, cbt, want_psi=True, want_y=True)
    assert rec.shape == (200, 50)
    # Section 4's count: one 16-bit number plus the code bits of all levels
    code_bits = 64 * 4 + 32 * 2 + 16 * 2 + 8 * 2 + 4 * bits[0] + 2 * bits[1] + bits[2]
    assert code_bits + 16 <= 50 * 8 and (50 * 8 - code_bits - 16) == 16 - (4 * bits[0] + 2 * bits[1] + bits[2])
    # levels 1..4 are the depth-4 record's (the recursion is open loop: every angle comes from exact radii)
    assert np.array_equal(rec[:, :46], oracle.encode(X0[:200], S, cb)[:, :46])
    J, rad = oracle.unpack_deep(rec, bits)
    assert np.array_equal(rad, np.linalg.norm(Y, axis=1).astype(np.float16).view(np.uint16))
    for i in range(0, 200, 7):
        p, r = oracle.polar(Y[i], 7)
        assert np.array_equal(p, psi[i]) and abs(r[0] - np.linalg.norm(Y[i])) <= 1e-12
        for l, (a0, a1) in {5: (120, 124), 6: (124, 126), 7: (126, 127)}.items():
            theta = cbt[l - 5, : 2 ** bits[l - 5]]
            assert np.array_equal(np.argmin(np.abs(theta[None, :] - p[a0:a1, None]), axis=1), J[i, a0:a1])
    # hand-unpacked code word of one record: little-endian 16 bits, level 5 first, lowest bits first
    word = int(rec[3, 46]) | (int(rec[3, 47]) << 8)
    got, pos = [], 0
    for l, n in ((5, 4), (6, 2), (7, 1)):
        for _ in range(n):
            got.append((word >> pos) & ((1 << bits[l - 5]) - 1))
            pos += bits[l - 5]
    assert got == list(J[3, 120:]) and word >> pos == 0
    assert int(rec[3, 48]) | (int(rec[3, 49]) << 8) == int(rad[3])


@pytest.mark.parametrize("bits", DEEP_BITS)
def test_deep_dequant_is_inverse_transform_of_centroids(S, cb, X0, bits):
    cbt = oracle.upper_codebooks(bits)
    rec = oracle.encode_deep(X0[:64], S, cb, bits, cbt)
    J, rad = oracle.unpack_deep(rec, bits)
    yhat = oracle.decode_deep(rec, S, cb, bits, cbt, rotated=True)
    r = rad.view(np.float16).astype(np.float64)
    # the whole vector lies on the sphere of the one stored radius
    assert np.max(np.abs(np.linalg.norm(yhat, axis=1) - r)) <= 1e-12
    # closed product form of Definition 1 (0-based): coordinate i takes cos at level l if bit l-1 of i is 0
    tables = [cb[0:16], cb[16:20], cb[20:24], cb[24:28], cbt[0], cbt[1], cbt[2]]
    offs = [0, 64, 96, 112, 120, 124, 126]
    for v in (0, 17, 63):
        for i in range(128):
            val = r[v]
            for l in range(1, 8):
                ang = tables[l - 1][J[v, offs[l - 1] + (i >> l)]]
                val *= math.cos(ang) if ((i >> (l - 1)) & 1) == 0 else math.sin(ang)
            assert abs(val - yhat[v, i]) <= 1e-12
    xhat = oracle.decode_deep(rec, S, cb, bits, cbt)
    assert np.max(np.abs(xhat - yhat @ S.T)) <= 1e-12
    # a zero vector stays zero
    z = oracle.encode_deep(np.zeros((1, 128)), S, cb, bits, cbt)
    assert np.all(oracle.unpack_deep(z, bits)[0] == 0) and np.all(oracle.decode_deep(z, S, cb, bits, cbt) == 0.0)


def test_deep_reconstruction_error_matches_per_level_prediction(S, cb, X0):
    bits = (2, 2, 2)
    cbt = oracle.upper_codebooks(bits)
    prod = 1.0
    for level in range(1, 8):
        K = oracle.CB_K[level] if level <= 4 else 2 ** bits[level - 5]
        c, b = oracle.codebook(level, K)
        m = 0 if level == 1 else 2 ** (level - 1) - 1
        pdf = lambda t: math.sin(2 * t) ** m if level > 1 else 1.0
        norm, _ = scipy.integrate.quad(pdf, b[0], b[-1], limit=200)
        prod *= sum(scipy.integrate.quad(lambda t, k=k: math.cos(t - c[k]) * pdf(t), b[k], b[k + 1], limit=200)[0]
                    for k in range(K)) / norm
    predicted = math.sqrt(2 * (1 - prod))
    xhat = oracle.decode_deep(oracle.encode_deep(X0, S, cb, bits, cbt), S, cb, bits, cbt)
    rel = np.linalg.norm(xhat - X0) / np.linalg.norm(X0)
    assert abs(rel - predicted) <= 0.004, (rel, predicted)
    # 3.11 bits per coordinate instead of 3.875 for a slightly larger error than depth 4
    assert 0.18 < rel < 0.20
    # more bits above level 4 can only help
    b3 = (3, 3, 3)   # 4*3 + 2*3 + 3 = 21 > 16: rejected
    with pytest.raises(AssertionError):
        oracle.upper_codebooks(b3)


def test_deep_attention_is_textbook_softmax(S, cb):
    bits = (2, 2, 2)
    cbt = oracle.upper_codebooks(bits)
    T, Hkv, B = 29, 2, 2
    k = synth.kv_stream(T * B, Hkv, 31).float().numpy().astype(np.float64)
    v = synth.kv_stream(T * B, Hkv, 32).float().numpy().astype(np.float64)
    k_rec = oracle.encode_deep(k.reshape(-1, 128), S, cb, bits, cbt).reshape(Hkv, T * B, 50)
    v_rec = oracle.encode_deep(v.reshape(-1, 128), S, cb, bits, cbt).reshape(Hkv, T * B, 50)
    q = synth.queries(B, 4 * Hkv, 33).float().numpy().astype(np.float64)
    seq_start = np.array([0, T], dtype=np.int64)
    ctx_len = np.array([T, 0], dtype=np.int32)
    scale = 1 / math.sqrt(128)
    out = oracle.attention_deep(q, k_rec, v_rec, seq_start, ctx_len, S, cb, bits, cbt, scale)
    assert np.all(out[1] == 0.0)
    for h in range(4 * Hkv):
        Kh = oracle.decode_deep(k_rec[h // 4, :T], S, cb, bits, cbt)
        Vh = oracle.decode_deep(v_rec[h // 4, :T], S, cb, bits, cbt)
        p = scipy.special.softmax(Kh @ q[0, h] * scale)
        assert np.max(np.abs(p @ Vh - out[0, h])) <= 1e-12


def test_deep_hybrid_attention_reductions(S, cb):
    """The numpy-written hybrid attention on deep records: an empty window is attention_deep, an empty prefix is
    plain softmax attention on the window, and the general case is the log-sum-exp merge of the two."""
    bits = (2, 2, 2)
    cbt = oracle.upper_codebooks(bits)
    T, W, Hkv, B = 23, 9, 2, 2
    k = synth.kv_stream(T * B, Hkv, 61).float().numpy().astype(np.float64)
    v = synth.kv_stream(T * B, Hkv, 62).float().numpy().astype(np.float64)
    k_rec = oracle.encode_deep(k.reshape(-1, 128), S, cb, bits, cbt).reshape(Hkv, T * B, 50)
    v_rec = oracle.encode_deep(v.reshape(-1, 128), S, cb, bits, cbt).reshape(Hkv, T * B, 50)
    wk = synth.kv_stream(B * W, Hkv, 63).float().numpy().astype(np.float64).reshape(Hkv, B, W, 128).transpose(1, 0, 2, 3)
    wv = synth.kv_stream(B * W, Hkv, 64).float().numpy().astype(np.float64).reshape(Hkv, B, W, 128).transpose(1, 0, 2, 3)
    q = synth.queries(B, 2 * Hkv, 65).float().numpy().astype(np.float64)
    starts, lens = np.array([0, T], np.int64), np.array([T, T - 4], np.int32)
    scale = 1 / math.sqrt(128)
    full = oracle.attention_hybrid_deep(q, k_rec, v_rec, starts, lens, wk, wv, np.array([W, W - 2]), S, cb, bits, cbt, scale)
    none = oracle.attention_hybrid_deep(q, k_rec, v_rec, starts, lens, wk, wv, np.array([0, 0]), S, cb, bits, cbt, scale)
    assert np.max(np.abs(none - oracle.attention_deep(q, k_rec, v_rec, starts, lens, S, cb, bits, cbt, scale))) <= 1e-12
    only = oracle.attention_hybrid_deep(q, k_rec, v_rec, starts, np.array([0, 0], np.int32), wk, wv, np.array([W, W - 2]), S, cb,
                                        bits, cbt, scale)
    for b, w in ((0, W), (1, W - 2)):
        for h in range(2 * Hkv):
            ref = oracle.attention_exact(q[b, h:h + 1], wk[b, h // 2, :w], wv[b, h // 2, :w], scale)[0]
            assert np.max(np.abs(only[b, h] - ref)) <= 1e-12
            # merge of the two parts with their log-sum-exp weights
            Kp = oracle.decode_deep(k_rec[h // 2, starts[b]:starts[b] + lens[b]], S, cb, bits, cbt)
            lse_p = scipy.special.logsumexp(Kp @ q[b, h] * scale)
            lse_w = scipy.special.logsumexp(wk[b, h // 2, :w] @ q[b, h] * scale)
            a = 1 / (1 + math.exp(lse_w - lse_p))
            assert np.max(np.abs(full[b, h] - (a * none[b, h] + (1 - a) * only[b, h]))) <= 1e-12


def test_stored_radius_saturates_at_the_largest_finite_binary16():
    """Section 4.1 stores radii in 16 bits and is silent on what lies beyond the format's range.  Reading: the stored
    radius saturates at 65504; the codes (the direction) are those of the exact vector, and DeQuant stays finite."""
    S, cb = oracle.preconditioner(0), oracle.default_codebooks()
    g = np.random.default_rng(5).standard_normal((4, 128))
    x = np.stack([g[0], 3e4 * g[1], 1e6 * g[2], g[3]])
    rec = oracle.encode(x, S, cb)
    J, r = oracle.unpack(rec)
    radii = r.view(np.float16).astype(np.float64)
    assert np.all(np.isfinite(radii))
    exact = np.linalg.norm((x @ S).reshape(4, 8, 16), axis=2)
    assert np.all(radii[1][exact[1] > 65520] == 65504.0) and np.all(radii[2] == 65504.0)
    small = exact < 65504
    assert np.allclose(radii[small], exact[small], rtol=2.0 ** -11)
    # the direction is unaffected by the scale: the codes of 1e6 * g equal those of g
    assert np.array_equal(J[2], oracle.unpack(oracle.encode(g[2:3], S, cb))[0][0])
    assert np.all(np.isfinite(oracle.decode(rec, S, cb)))
    for bits in ((2, 2, 2),):
        cbt = oracle.upper_codebooks(bits)
        rec7 = oracle.encode_deep(x, S, cb, bits, cbt)
        _, r7 = oracle.unpack_deep(rec7, bits)
        r7 = r7.view(np.float16).astype(np.float64)
        assert r7[2] == 65504.0 and np.isclose(r7[0], np.linalg.norm(g[0]), rtol=2.0 ** -11)


def test_tie_rule_boundaries_follow_the_codebooks_in_use():
    """The GPU tests accept a differing code only next to a cell boundary of Quant (nearest centroid): the helper
    that measures that distance, given the analytic centroids as data, must place the boundaries where the
    analytic codebooks' own boundaries are, and with moved centroids at the middles between neighbours."""
    from tests import helpers

    rng = np.random.default_rng(5)
    psi = np.concatenate([rng.uniform(0, 2 * np.pi, (50, 64)), rng.uniform(0, np.pi / 2, (50, 56))], axis=1)
    cb = oracle.default_codebooks()
    assert np.allclose(helpers.boundary_distance(psi, cb), helpers.boundary_distance(psi), atol=1e-12)
    moved = cb.copy()
    moved[3] += 0.05          # level-1 centroid 3: its two boundaries move by 0.025
    moved[17] -= 0.02         # level-2 centroid 1
    at = np.zeros((1, 120))
    at[0, 0] = 0.5 * (moved[3] + moved[4])
    at[0, 64] = 0.5 * (moved[16] + moved[17])
    d = helpers.boundary_distance(at, moved)
    assert d[0, 0] <= 1e-15 and d[0, 64] <= 1e-15
    assert helpers.boundary_distance(at, cb)[0, 0] > 0.02 and helpers.boundary_distance(at, cb)[0, 64] > 0.005
    # and the oracle's Quant does switch cells exactly there
    for col, lvl_slice, mid in ((0, slice(0, 16), at[0, 0]), (64, slice(16, 20), at[0, 64])):
        c = moved[lvl_slice]
        lo = int(np.argmin(np.abs(mid - 1e-9 - c))), int(np.argmin(np.abs(mid + 1e-9 - c)))
        assert lo[1] == lo[0] + 1
