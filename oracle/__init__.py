"""fp64 CPU oracle for the PolarQuant hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``pq_oracle.c`` (plain C, double precision).  Only
tests, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may
import this package.  It shares no code with the HIP library and never
imports it.

All array arguments are numpy arrays; inputs are widened to float64 by the
caller (bf16/fp32 widen exactly).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pq_oracle.c")
_LIB = os.path.join(_HERE, "libpq_oracle.so")

D = 128
NANG = 120
NBLK = 8
REC = 62
CB_LEN = 28
CB_OFF = {1: 0, 2: 16, 3: 20, 4: 24}
CB_K = {1: 16, 2: 4, 3: 4, 4: 4}


def build(force=False):
    """Compile the oracle with gcc -O2 (OpenMP over independent units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c_dp = ctypes.POINTER(ctypes.c_double)
        L.orc_angle_pdf.restype = ctypes.c_double
        L.orc_angle_pdf.argtypes = [ctypes.c_int, ctypes.c_double]
        L.orc_codebook_distortion.restype = ctypes.c_double
        L.orc_codebook_distortion.argtypes = [ctypes.c_int, ctypes.c_int, c_dp]
        L.orc_f64_to_f16.restype = ctypes.c_uint16
        L.orc_f64_to_f16.argtypes = [ctypes.c_double]
        L.orc_f16_to_f64.restype = ctypes.c_double
        L.orc_f16_to_f64.argtypes = [ctypes.c_uint16]
        L.orc_quant.restype = ctypes.c_int
        L.orc_quant.argtypes = [ctypes.c_double, c_dp, ctypes.c_int]
        L.orc_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a, ty=ctypes.c_double):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads():
    return int(lib().orc_num_threads())


def gaussian_matrix(seed, d=D):
    G = np.empty((d, d), dtype=np.float64)
    lib().orc_gaussian_matrix(ctypes.c_uint64(seed), ctypes.c_int(d), _p(G))
    return G


def rotation_from_gaussian(G):
    G = _f64(G)
    d = G.shape[0]
    S = np.empty((d, d), dtype=np.float64)
    rc = lib().orc_rotation_from_gaussian(_p(G), ctypes.c_int(d), _p(S))
    assert rc == 0
    return S


def preconditioner(seed, d=D):
    """S of Section 4.1: rotation from the QR of the seeded Gaussian matrix."""
    return rotation_from_gaussian(gaussian_matrix(seed, d))


def angle_pdf(level, psi):
    return float(lib().orc_angle_pdf(int(level), float(psi)))


def codebook(level, K):
    c = np.empty(K, dtype=np.float64)
    b = np.empty(K + 1, dtype=np.float64)
    rc = lib().orc_codebook(ctypes.c_int(level), ctypes.c_int(K), _p(c), _p(b))
    assert rc == 0
    return c, b


def codebook_distortion(level, centroids):
    c = _f64(centroids)
    return float(lib().orc_codebook_distortion(int(level), int(c.size), _p(c)))


def default_codebooks():
    cb = np.empty(CB_LEN, dtype=np.float64)
    rc = lib().orc_default_codebooks(_p(cb))
    assert rc == 0
    return cb


def polar(y, L):
    y = _f64(y)
    d = y.size
    nang = sum(d >> l for l in range(1, L + 1))
    psi = np.empty(nang, dtype=np.float64)
    r = np.empty(d >> L, dtype=np.float64)
    lib().orc_polar(_p(y), ctypes.c_int(d), ctypes.c_int(L), _p(psi), _p(r))
    return psi, r


def polar_inverse(psi, r, d, L):
    psi = _f64(psi)
    r = _f64(r)
    y = np.empty(d, dtype=np.float64)
    lib().orc_polar_inverse(_p(psi), _p(r), ctypes.c_int(d), ctypes.c_int(L), _p(y))
    return y


def quant(psi, theta):
    theta = _f64(theta)
    return int(lib().orc_quant(float(psi), _p(theta), int(theta.size)))


def f64_to_f16(x):
    return int(lib().orc_f64_to_f16(float(x)))


def f16_to_f64(h):
    return float(lib().orc_f16_to_f64(int(h)))


def pack(J, rad):
    J = np.ascontiguousarray(J, dtype=np.int32)
    rad = np.ascontiguousarray(rad, dtype=np.uint16)
    n = J.shape[0]
    rec = np.empty((n, REC), dtype=np.uint8)
    lib().orc_pack(_p(J, ctypes.c_int32), _p(rad, ctypes.c_uint16), ctypes.c_int64(n), _p(rec, ctypes.c_uint8))
    return rec


def unpack(rec):
    rec = np.ascontiguousarray(rec, dtype=np.uint8)
    n = rec.shape[0]
    J = np.empty((n, NANG), dtype=np.int32)
    rad = np.empty((n, NBLK), dtype=np.uint16)
    lib().orc_unpack(_p(rec, ctypes.c_uint8), ctypes.c_int64(n), _p(J, ctypes.c_int32), _p(rad, ctypes.c_uint16))
    return J, rad


def encode(x, S, cb, want_psi=False, want_y=False):
    """x[n,128] -> canonical records [n,62] (+ exact angles / rotated vectors)."""
    x = _f64(x).reshape(-1, D)
    S = _f64(S)
    cb = _f64(cb)
    n = x.shape[0]
    rec = np.empty((n, REC), dtype=np.uint8)
    psi = np.empty((n, NANG), dtype=np.float64) if want_psi else None
    y = np.empty((n, D), dtype=np.float64) if want_y else None
    lib().orc_encode(
        _p(x), ctypes.c_int64(n), _p(S), _p(cb), _p(rec, ctypes.c_uint8),
        _p(psi) if want_psi else None, _p(y) if want_y else None,
    )
    out = [rec]
    if want_psi:
        out.append(psi)
    if want_y:
        out.append(y)
    return out[0] if len(out) == 1 else tuple(out)


def decode(rec, S, cb, rotated=False):
    rec = np.ascontiguousarray(rec, dtype=np.uint8).reshape(-1, REC)
    S = _f64(S)
    cb = _f64(cb)
    n = rec.shape[0]
    out = np.empty((n, D), dtype=np.float64)
    lib().orc_decode(_p(rec, ctypes.c_uint8), ctypes.c_int64(n), _p(S), _p(cb), ctypes.c_int(1 if rotated else 0), _p(out))
    return out


def attention(q, k_rec, v_rec, seq_start, ctx_len, S, cb, scale, rotated=False):
    """q[B,Hq,128]; k_rec/v_rec [Hkv, plane_tokens, 62] -> out[B,Hq,128] (float64)."""
    q = _f64(q)
    B, Hq, _ = q.shape
    k_rec = np.ascontiguousarray(k_rec, dtype=np.uint8)
    v_rec = np.ascontiguousarray(v_rec, dtype=np.uint8)
    Hkv, plane, _ = k_rec.shape
    assert v_rec.shape == k_rec.shape and Hq % Hkv == 0
    seq_start = np.ascontiguousarray(seq_start, dtype=np.int64)
    ctx_len = np.ascontiguousarray(ctx_len, dtype=np.int32)
    assert seq_start.size == B and ctx_len.size == B
    assert np.all(seq_start + ctx_len <= plane)
    S = _f64(S)
    cb = _f64(cb)
    out = np.empty((B, Hq, D), dtype=np.float64)
    lib().orc_attention(
        _p(q), ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(Hkv),
        _p(k_rec, ctypes.c_uint8), _p(v_rec, ctypes.c_uint8),
        _p(seq_start, ctypes.c_int64), _p(ctx_len, ctypes.c_int32),
        ctypes.c_int64(plane), _p(S), _p(cb), ctypes.c_double(scale),
        ctypes.c_int(1 if rotated else 0), _p(out),
    )
    return out


def attention_hybrid(q, k_rec, v_rec, seq_start, ctx_len, win_k, win_v, win_len, S, cb, scale):
    """Quantised prefix + unquantised window: q[B,Hq,128]; k_rec/v_rec [Hkv, plane, 62];
    win_k/win_v [B, Hkv, win_cap, 128]; win_len [B] -> out[B,Hq,128] (float64)."""
    q = _f64(q)
    B, Hq, _ = q.shape
    k_rec = np.ascontiguousarray(k_rec, dtype=np.uint8)
    v_rec = np.ascontiguousarray(v_rec, dtype=np.uint8)
    Hkv, plane, _ = k_rec.shape
    assert v_rec.shape == k_rec.shape and Hq % Hkv == 0
    seq_start = np.ascontiguousarray(seq_start, dtype=np.int64)
    ctx_len = np.ascontiguousarray(ctx_len, dtype=np.int32)
    win_len = np.ascontiguousarray(win_len, dtype=np.int32)
    win_k = _f64(win_k)
    win_v = _f64(win_v)
    assert win_k.shape == win_v.shape and win_k.shape[:2] == (B, Hkv) and win_k.shape[3] == D
    cap = win_k.shape[2]
    assert seq_start.size == B and ctx_len.size == B and win_len.size == B
    assert np.all(seq_start + ctx_len <= plane) and np.all(win_len <= cap)
    S = _f64(S)
    cb = _f64(cb)
    out = np.empty((B, Hq, D), dtype=np.float64)
    lib().orc_attention_hybrid(
        _p(q), ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(Hkv),
        _p(k_rec, ctypes.c_uint8), _p(v_rec, ctypes.c_uint8),
        _p(seq_start, ctypes.c_int64), _p(ctx_len, ctypes.c_int32), ctypes.c_int64(plane),
        _p(win_k), _p(win_v), _p(win_len, ctypes.c_int32), ctypes.c_int64(cap),
        _p(S), _p(cb), ctypes.c_double(scale), _p(out),
    )
    return out


def fit_codebooks(x, S, cb_init, iterations):
    """Online codebooks: `iterations` k-means (Lloyd) rounds on the angles of x[n,128] rotated by S,
    from the 28 centroids cb_init -> 28 centroids."""
    x = _f64(x).reshape(-1, D)
    S = _f64(S)
    cb_init = _f64(cb_init).reshape(-1)
    assert cb_init.size == 28
    out = np.empty(28, dtype=np.float64)
    lib().orc_fit_codebooks(_p(x), ctypes.c_int64(x.shape[0]), _p(S), _p(cb_init), ctypes.c_int(int(iterations)), _p(out))
    return out


def attention_exact(q, K, V, scale):
    """Plain softmax attention on unquantised K,V[T,128] for q[G,128] (reporting only)."""
    q = _f64(q).reshape(-1, D)
    K = _f64(K)
    V = _f64(V)
    out = np.empty_like(q)
    lib().orc_attention_exact(_p(q), _p(K), _p(V), ctypes.c_int64(K.shape[0]), ctypes.c_int(q.shape[0]), ctypes.c_double(scale), _p(out))
    return out


# ---- full-depth recursion (L = 7): one radius per vector, 50-byte records ----
REC_DEEP = 50
NANG_DEEP = 127


def _bits(bits):
    b = np.ascontiguousarray(bits, dtype=np.int32).reshape(-1)
    assert b.size == 3
    return b


def upper_codebooks(bits):
    """Lloyd-Max codebooks of levels 5, 6, 7 with 2^bits[l-5] centroids: array [3, 8] (unused entries 0)."""
    b = _bits(bits)
    cbt = np.zeros((3, 8), dtype=np.float64)
    rc = lib().orc_upper_codebooks(_p(b, ctypes.c_int32), _p(cbt))
    assert rc == 0, "bits must be 1..3 each with 4 b5 + 2 b6 + b7 <= 16"
    return cbt


def fit_upper_codebooks(x, S, bits, cbt_init, iterations):
    """Online codebooks of levels 5, 6, 7 (Section 4.1's k-means on the data's own angles, at the levels
    that Definition 1 adds above level 4): `iterations` Lloyd rounds per level on the exact angles of
    x[n,128] rotated by S, from the centroids cbt_init[3,8] (2^bits[l-5] used per row) -> [3,8].
    Nearest centroid by linear distance, the lower cell on a tie; a centroid with an empty cell stays."""
    b = _bits(bits)
    cbt = _f64(cbt_init).reshape(3, 8).copy()
    x = _f64(x).reshape(-1, D)
    _, psi, _ = encode_deep(x, S, default_codebooks(), b, upper_codebooks(b), want_psi=True, want_y=True)
    psi = psi.reshape(-1, NANG_DEEP)
    cols = ((120, 124), (124, 126), (126, 127))
    for l in range(3):
        K = 1 << int(b[l])
        samples = np.sort(psi[:, cols[l][0]:cols[l][1]].reshape(-1))
        c = cbt[l, :K].copy()
        for _ in range(int(iterations)):
            edges = 0.5 * (c[:-1] + c[1:])
            cell = np.searchsorted(edges, samples, side="left")
            for k in range(K):
                mine = samples[cell == k]
                if mine.size:
                    c[k] = mine.mean()
        cbt[l, :K] = c
    return cbt


def unpack_deep(rec, bits):
    rec = np.ascontiguousarray(rec, dtype=np.uint8).reshape(-1, REC_DEEP)
    b = _bits(bits)
    n = rec.shape[0]
    J = np.empty((n, NANG_DEEP), dtype=np.int32)
    rad = np.empty(n, dtype=np.uint16)
    lib().orc_unpack_deep(_p(rec, ctypes.c_uint8), ctypes.c_int64(n), _p(b, ctypes.c_int32), _p(J, ctypes.c_int32),
                          _p(rad, ctypes.c_uint16))
    return J, rad


def encode_deep(x, S, cb, bits, cbt, want_psi=False, want_y=False):
    """x[n,128] -> deep records [n,50] (+ the 127 exact angles / rotated vectors)."""
    x = _f64(x).reshape(-1, D)
    S = _f64(S)
    cb = _f64(cb)
    b = _bits(bits)
    cbt = _f64(cbt).reshape(3, 8)
    n = x.shape[0]
    rec = np.empty((n, REC_DEEP), dtype=np.uint8)
    psi = np.empty((n, NANG_DEEP), dtype=np.float64) if want_psi else None
    y = np.empty((n, D), dtype=np.float64) if want_y else None
    lib().orc_encode_deep(
        _p(x), ctypes.c_int64(n), _p(S), _p(cb), _p(b, ctypes.c_int32), _p(cbt), _p(rec, ctypes.c_uint8),
        _p(psi) if want_psi else None, _p(y) if want_y else None,
    )
    out = [rec]
    if want_psi:
        out.append(psi)
    if want_y:
        out.append(y)
    return out[0] if len(out) == 1 else tuple(out)


def decode_deep(rec, S, cb, bits, cbt, rotated=False):
    rec = np.ascontiguousarray(rec, dtype=np.uint8).reshape(-1, REC_DEEP)
    S = _f64(S)
    cb = _f64(cb)
    b = _bits(bits)
    cbt = _f64(cbt).reshape(3, 8)
    n = rec.shape[0]
    out = np.empty((n, D), dtype=np.float64)
    lib().orc_decode_deep(_p(rec, ctypes.c_uint8), ctypes.c_int64(n), _p(S), _p(cb), _p(b, ctypes.c_int32), _p(cbt),
                          ctypes.c_int(1 if rotated else 0), _p(out))
    return out


def attention_deep(q, k_rec, v_rec, seq_start, ctx_len, S, cb, bits, cbt, scale):
    """q[B,Hq,128]; k_rec/v_rec [Hkv, plane_tokens, 50] -> out[B,Hq,128] (float64)."""
    q = _f64(q)
    B, Hq, _ = q.shape
    k_rec = np.ascontiguousarray(k_rec, dtype=np.uint8)
    v_rec = np.ascontiguousarray(v_rec, dtype=np.uint8)
    Hkv, plane, rb = k_rec.shape
    assert rb == REC_DEEP and v_rec.shape == k_rec.shape and Hq % Hkv == 0
    seq_start = np.ascontiguousarray(seq_start, dtype=np.int64)
    ctx_len = np.ascontiguousarray(ctx_len, dtype=np.int32)
    assert seq_start.size == B and ctx_len.size == B
    assert np.all(seq_start + ctx_len <= plane)
    S = _f64(S)
    cb = _f64(cb)
    b = _bits(bits)
    cbt = _f64(cbt).reshape(3, 8)
    out = np.empty((B, Hq, D), dtype=np.float64)
    lib().orc_attention_deep(
        _p(q), ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(Hkv),
        _p(k_rec, ctypes.c_uint8), _p(v_rec, ctypes.c_uint8),
        _p(seq_start, ctypes.c_int64), _p(ctx_len, ctypes.c_int32),
        ctypes.c_int64(plane), _p(S), _p(cb), _p(b, ctypes.c_int32), _p(cbt), ctypes.c_double(scale), _p(out),
    )
    return out


def attention_hybrid_deep(q, k_rec, v_rec, seq_start, ctx_len, win_k, win_v, win_len, S, cb, bits, cbt, scale):
    """Deep-record prefix + unquantised window, one softmax over both (Eq. 5 with the rows of the window appended
    as given; Section 5.3).  The definition written out with numpy in float64: DeQuant of the prefix rows, the
    window rows appended, scores, exp of the shifted scores, normalised weighted sum.
    q[B,Hq,128]; k_rec/v_rec [Hkv, plane, 50]; win_k/win_v [B, Hkv, win_cap, 128]; win_len [B] -> [B,Hq,128]."""
    q = _f64(q)
    B, Hq, _ = q.shape
    Hkv = k_rec.shape[0]
    G = Hq // Hkv
    win_k = _f64(win_k)
    win_v = _f64(win_v)
    out = np.zeros((B, Hq, D), dtype=np.float64)
    for b in range(B):
        T, W = max(int(ctx_len[b]), 0), max(int(win_len[b]), 0)
        if T + W == 0:
            continue
        s0 = int(seq_start[b])
        for hk in range(Hkv):
            Kh = np.concatenate([decode_deep(k_rec[hk, s0:s0 + T], S, cb, bits, cbt) if T else np.zeros((0, D)), win_k[b, hk, :W]])
            Vh = np.concatenate([decode_deep(v_rec[hk, s0:s0 + T], S, cb, bits, cbt) if T else np.zeros((0, D)), win_v[b, hk, :W]])
            for g in range(G):
                s = Kh @ q[b, hk * G + g] * scale
                p = np.exp(s - s.max())
                out[b, hk * G + g] = (p / p.sum()) @ Vh
    return out


# ---- general format: any depth 1..7, any bits per level (remark after Theorem 1; Definition 1) ----
def _gbits(bits):
    b = np.ascontiguousarray(bits, dtype=np.int32)
    return b, b.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def general_nang(L):
    return sum(D >> l for l in range(1, L + 1))


def general_record_bytes(L, bits):
    b, bp = _gbits(bits)
    n = lib().orc_general_record_bytes(ctypes.c_int(L), bp)
    if n < 0:
        raise ValueError("bad depth or bits")
    return int(n)


def general_codebooks(L, bits):
    """Lloyd-Max centroids of levels 1..L, concatenated (level l: 2^bits[l-1] entries)."""
    b, bp = _gbits(bits)
    out = np.zeros(sum(1 << int(w) for w in b[:L]), dtype=np.float64)
    if lib().orc_general_codebooks(ctypes.c_int(L), bp, _p(out)):
        raise RuntimeError("codebook iteration failed")
    return out


def encode_general(x, S, L, bits, cbg, want_psi=False, want_codes=False):
    x = _f64(x).reshape(-1, D)
    S, cbg = _f64(S), _f64(cbg)
    b, bp = _gbits(bits)
    n, rb, nang = x.shape[0], general_record_bytes(L, bits), general_nang(L)
    rec = np.zeros((n, rb), dtype=np.uint8)
    psi = np.zeros((n, nang), dtype=np.float64) if want_psi else None
    J = np.zeros((n, nang), dtype=np.int32) if want_codes else None
    lib().orc_encode_general(_p(x), ctypes.c_int64(n), _p(S), ctypes.c_int(L), bp, _p(cbg), _p(rec, ctypes.c_uint8),
                             _p(psi) if want_psi else None, _p(J, ctypes.c_int32) if want_codes else None)
    res = [rec]
    if want_psi:
        res.append(psi)
    if want_codes:
        res.append(J)
    return res[0] if len(res) == 1 else tuple(res)


def decode_general(rec, S, L, bits, cbg, rotated=False):
    rb = general_record_bytes(L, bits)
    rec = np.ascontiguousarray(rec, dtype=np.uint8).reshape(-1, rb)
    S, cbg = _f64(S), _f64(cbg)
    b, bp = _gbits(bits)
    out = np.zeros((rec.shape[0], D), dtype=np.float64)
    lib().orc_decode_general(_p(rec, ctypes.c_uint8), ctypes.c_int64(rec.shape[0]), _p(S), ctypes.c_int(L), bp, _p(cbg),
                             ctypes.c_int(1 if rotated else 0), _p(out))
    return out


def attention_general(q, k_rec, v_rec, seq_start, ctx_len, S, L, bits, cbg, scale):
    """q [B, Hq, 128]; k_rec, v_rec [Hkv, plane_tokens, record bytes]."""
    q = _f64(q)
    B, Hq, _ = q.shape
    k_rec = np.ascontiguousarray(k_rec, dtype=np.uint8)
    v_rec = np.ascontiguousarray(v_rec, dtype=np.uint8)
    Hkv, plane = k_rec.shape[0], k_rec.shape[1]
    S, cbg = _f64(S), _f64(cbg)
    b, bp = _gbits(bits)
    ss = np.ascontiguousarray(seq_start, dtype=np.int64)
    cl = np.ascontiguousarray(ctx_len, dtype=np.int32)
    out = np.zeros((B, Hq, D), dtype=np.float64)
    lib().orc_attention_general(_p(q), ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(Hkv), _p(k_rec, ctypes.c_uint8),
                                _p(v_rec, ctypes.c_uint8), _p(ss, ctypes.c_int64), _p(cl, ctypes.c_int32),
                                ctypes.c_int64(plane), _p(S), ctypes.c_int(L), bp, _p(cbg), ctypes.c_double(scale), _p(out))
    return out
