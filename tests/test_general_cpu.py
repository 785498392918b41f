"""CPU pins of the oracle's general format (any recursion depth, any bits per level: Definition 1 and the remark
after Theorem 1; Section 4.1 is the instance depth 4, bits 4/2/2/2)."""
import math

import numpy as np
import pytest
from scipy import integrate, special

import oracle

D = 128


def gaussian(n, seed):
    return np.random.default_rng(seed).standard_normal((n, D))


def python_bit_stream(codes_by_level, bits):
    """Independent writer of the record's code part: little-endian bit stream, level after level."""
    out = []
    for codes, w in zip(codes_by_level, bits):
        for c in codes:
            out.extend((int(c) >> i) & 1 for i in range(w))
    out.extend([0] * (-len(out) % 8))
    return np.packbits(np.array(out, dtype=np.uint8).reshape(-1, 8), axis=1, bitorder="little").reshape(-1)


def test_general_format_with_section_4_1_settings_is_the_section_4_1_path():
    S, cb = oracle.preconditioner(3), oracle.default_codebooks()
    bits = [4, 2, 2, 2]
    cbg = oracle.general_codebooks(4, bits)
    assert np.array_equal(cbg, cb)
    x = gaussian(300, 1)
    x[:, [3, 70]] *= 9.0
    rec_g, psi_g, J_g = oracle.encode_general(x, S, 4, bits, cbg, want_psi=True, want_codes=True)
    rec, psi = oracle.encode(x, S, cb, want_psi=True)
    J, rad = oracle.unpack(rec)
    assert np.array_equal(psi_g, psi) and np.array_equal(J_g, J)
    assert np.array_equal(rec_g[:, 46:].view(np.uint16), rad.astype(np.uint16))      # the 8 block radii
    assert np.array_equal(oracle.decode_general(rec_g, S, 4, bits, cbg), oracle.decode(rec, S, cb))
    assert np.array_equal(oracle.decode_general(rec_g, S, 4, bits, cbg, rotated=True), oracle.decode(rec, S, cb, rotated=True))


@pytest.mark.parametrize("L,bits,nbytes", [(4, [3, 3, 2, 3], 43 + 16), (5, [4, 2, 2, 2, 2], 47 + 8),
                                            (6, [4, 2, 2, 2, 2, 3], 48 + 4), (7, [3, 2, 3, 2, 1, 2, 3], 42 + 2)])
def test_general_record_size_and_bit_order(L, bits, nbytes):
    assert oracle.general_record_bytes(L, bits) == nbytes
    S = oracle.preconditioner(5)
    cbg = oracle.general_codebooks(L, bits)
    x = gaussian(40, 2)
    rec, psi, J = oracle.encode_general(x, S, L, bits, cbg, want_psi=True, want_codes=True)
    y = x @ S
    psi_ref, r_ref = zip(*(oracle.polar(row, L) for row in y))
    assert np.allclose(psi, np.array(psi_ref), atol=1e-11, rtol=0)   # numpy sums the rotation in another order
    for i in range(x.shape[0]):
        levels, off = [], 0
        for l in range(1, L + 1):
            n = D >> l
            levels.append(J[i, off:off + n])
            assert J[i, off:off + n].max() < (1 << bits[l - 1])
            off += n
        code_part = python_bit_stream(levels, bits)
        assert np.array_equal(rec[i, :len(code_part)], code_part)
        radii = rec[i, len(code_part):].view(np.uint16)
        assert len(radii) == D >> L
        assert np.array_equal(radii, np.array(r_ref[i]).astype(np.float16).view(np.uint16))
    # codes are nearest centroids (brute force), level by level
    off, cboff = 0, 0
    for l in range(1, L + 1):
        n, K = D >> l, 1 << bits[l - 1]
        c = cbg[cboff:cboff + K]
        assert np.array_equal(J[:, off:off + n], np.argmin(np.abs(psi[:, off:off + n, None] - c), axis=2))
        off, cboff = off + n, cboff + K


@pytest.mark.parametrize("level,K", [(1, 8), (2, 8), (3, 8), (4, 8), (5, 4), (6, 8)])
def test_general_codebooks_satisfy_the_lloyd_max_conditions(level, K):
    """Centroid = conditional mean of its cell under Lemma 2's density, cell boundaries = midpoints (Eq. 3's
    stationarity), re-checked with scipy quadrature of sin^(2^(l-1) - 1)(2 psi)."""
    bits = [3] * 7
    bits[level - 1] = int(math.log2(K))
    cbg = oracle.general_codebooks(level, bits[:level])
    c = cbg[-K:]
    if level == 1:
        assert np.allclose(c, (np.arange(K) + 0.5) * 2 * math.pi / K, rtol=0, atol=1e-15)
        return
    m = 2 ** (level - 1) - 1
    pdf = lambda t: math.sin(2 * t) ** m
    edges = np.concatenate([[0.0], 0.5 * (c[1:] + c[:-1]), [math.pi / 2]])
    assert np.all(np.diff(c) > 0) and np.allclose(c + c[::-1], math.pi / 2, atol=1e-12)   # symmetric about pi/4
    for k in range(K):
        m0 = integrate.quad(pdf, edges[k], edges[k + 1], epsabs=1e-15, epsrel=1e-13)[0]
        m1 = integrate.quad(lambda t: t * pdf(t), edges[k], edges[k + 1], epsabs=1e-15, epsrel=1e-13)[0]
        assert abs(m1 / m0 - c[k]) < 1e-10


@pytest.mark.parametrize("L,bits", [(5, [4, 2, 2, 2, 2]), (6, [3, 3, 3, 2, 2, 2]), (7, [4, 3, 2, 2, 1, 1, 1])])
def test_general_depths_store_the_right_radii_and_keep_the_vector_on_its_sphere(L, bits):
    S = oracle.preconditioner(6)
    cbg = oracle.general_codebooks(L, bits)
    x = gaussian(500, 4)
    rec = oracle.encode_general(x, S, L, bits, cbg)
    y = x @ S
    nrad = D >> L
    radii = rec[:, -2 * nrad:].copy().view(np.float16).astype(np.float64)
    group = y.reshape(-1, nrad, D // nrad)
    assert np.allclose(radii, np.linalg.norm(group, axis=2), rtol=2 ** -11)               # r^(L) = group norms, binary16
    yhat = oracle.decode_general(rec, S, L, bits, cbg, rotated=True)
    assert np.allclose(np.linalg.norm(yhat.reshape(-1, nrad, D // nrad), axis=2), radii, rtol=1e-12)
    xhat = oracle.decode_general(rec, S, L, bits, cbg)
    assert np.allclose(xhat @ S, yhat, atol=1e-12)
    # relative reconstruction error against the per-level prediction sqrt(2 (1 - prod_l E cos delta_l)), with
    # E cos delta_l measured on the exact angles and their centroids
    rec2, psi, J = oracle.encode_general(x, S, L, bits, cbg, want_psi=True, want_codes=True)
    off, cboff, prod = 0, 0, 1.0
    for l in range(1, L + 1):
        n, K = D >> l, 1 << bits[l - 1]
        prod *= np.mean(np.cos(psi[:, off:off + n] - cbg[cboff:cboff + K][J[:, off:off + n]]))
        off, cboff = off + n, cboff + K
    err = np.linalg.norm(xhat - x) / np.linalg.norm(x)
    assert abs(err - math.sqrt(2 * (1 - prod))) < 0.01


def test_more_bits_give_a_smaller_error_and_more_bytes():
    S = oracle.preconditioner(7)
    x = gaussian(400, 5)
    errs, sizes = [], []
    for bits in ([3, 2, 2, 2], [4, 2, 2, 2], [4, 3, 2, 2], [4, 3, 3, 3]):
        cbg = oracle.general_codebooks(4, bits)
        rec = oracle.encode_general(x, S, 4, bits, cbg)
        errs.append(np.linalg.norm(oracle.decode_general(rec, S, 4, bits, cbg) - x) / np.linalg.norm(x))
        sizes.append(rec.shape[1])
    assert errs[0] > errs[1] > errs[2] > errs[3] and sizes == sorted(sizes)


def test_general_attention_is_the_textbook_softmax_on_dequantised_rows():
    L, bits = 6, [3, 3, 2, 2, 2, 2]
    S = oracle.preconditioner(8)
    cbg = oracle.general_codebooks(L, bits)
    rb = oracle.general_record_bytes(L, bits)
    Hkv, Hq, lens = 2, 4, [5, 0, 37]
    plane = 64
    starts = np.array([0, 8, 16], dtype=np.int64)
    rng = np.random.default_rng(9)
    k_rec = np.zeros((Hkv, plane, rb), dtype=np.uint8)
    v_rec = np.zeros((Hkv, plane, rb), dtype=np.uint8)
    for h in range(Hkv):
        k_rec[h, :60] = oracle.encode_general(rng.standard_normal((60, D)), S, L, bits, cbg)
        v_rec[h, :60] = oracle.encode_general(rng.standard_normal((60, D)), S, L, bits, cbg)
    q = rng.standard_normal((3, Hq, D))
    scale = 1 / math.sqrt(D)
    got = oracle.attention_general(q, k_rec, v_rec, starts, lens, S, L, bits, cbg, scale)
    assert np.all(got[1] == 0)
    for b, n in enumerate(lens):
        for h in range(Hq):
            if n == 0:
                continue
            K = oracle.decode_general(k_rec[h // 2, starts[b]:starts[b] + n], S, L, bits, cbg)
            V = oracle.decode_general(v_rec[h // 2, starts[b]:starts[b] + n], S, L, bits, cbg)
            w = special.softmax(K @ q[b, h] * scale)
            assert np.allclose(got[b, h], w @ V, atol=1e-12)
