"""Shared helpers of the GPU parity tests: acceptance rules written out once.

Acceptance rules:
  codes   bit-exact against the fp64 oracle, except where the oracle's exact angle
          lies within 1e-5 rad of a codebook boundary; there the neighbouring code
          is accepted; overall mismatch rate <= 1e-4
  radii   bit-exact binary16, except where the oracle's exact radius lies within
          a relative 1e-6 of a binary16 rounding boundary; there +-1 ulp is
          accepted; overall mismatch rate <= 2e-3
  DeQuant <= 1e-3 relative L2
  attention <= 2e-3 relative L2 (bf16 inputs and outputs)
"""
import math

import numpy as np

import oracle
from tests import layout_ref

ANGLE_TOL = 1e-5
CODE_MISMATCH_RATE = 1e-4
RADIUS_REL_TOL = 1e-6
RADIUS_MISMATCH_RATE = 2e-3

_LEVEL_OF = np.concatenate([np.full(64, 1), np.full(32, 2), np.full(16, 3), np.full(8, 4)])


def boundary_distance(psi, cb=None):
    """psi [n,120] exact oracle angles -> distance to the nearest code boundary.  cb: the 28 centroids in use
    (16 of level 1, 4 each of levels 2-4) when they are not the analytic ones; a boundary is the middle between two
    neighbouring centroids (Quant takes the nearest centroid), and at level 1 also the seam 0 = 2 pi of the angle."""
    dist = np.empty_like(psi)
    a = psi[:, :64]
    if cb is None:
        step = np.pi / 8
        dist[:, :64] = np.abs(a - np.round(a / step) * step)
    else:
        c1 = np.asarray(cb[:16], dtype=np.float64)
        marks = np.concatenate([[0.0], 0.5 * (c1[:-1] + c1[1:]), [2.0 * np.pi]])
        dist[:, :64] = np.min(np.abs(a[..., None] - marks), axis=-1)
    off = 64
    for level, cnt in ((2, 32), (3, 16), (4, 8)):
        if cb is None:
            _, bnd = oracle.codebook(level, 4)
            inner = bnd[1:4]
        else:
            c = np.asarray(cb[16 + 4 * (level - 2) : 20 + 4 * (level - 2)], dtype=np.float64)
            inner = 0.5 * (c[:-1] + c[1:])
        a = psi[:, off : off + cnt]
        dist[:, off : off + cnt] = np.min(np.abs(a[..., None] - inner), axis=-1)
        off += cnt
    return dist


def check_codes(rec_gpu, rec_oracle, psi, enforce_rate=True, cb=None):
    """Returns a dict of statistics; raises AssertionError when the acceptance rule fails.
    enforce_rate=False leaves the rate limit to the caller, who pools the counts of several small calls
    (on a few hundred angles one legitimate tie already exceeds the rate).  cb: the centroids in use when they are
    not the analytic ones (the boundaries a mismatch must lie next to are theirs)."""
    Jg, rg = layout_ref.unpack_canonical(rec_gpu)   # the library's records never pass through the oracle package
    Jo, ro = oracle.unpack(rec_oracle)
    bad = Jg != Jo
    n_bad = int(bad.sum())
    stats = {"angles": int(Jo.size), "code_mismatches": n_bad, "code_mismatch_rate": n_bad / Jo.size}
    if n_bad:
        dist = boundary_distance(psi, cb)
        worst = float(dist[bad].max())
        stats["worst_mismatch_boundary_distance"] = worst
        assert worst <= ANGLE_TOL, f"code mismatch {worst:.3e} rad away from any boundary"
        diff = np.abs(Jg[bad].astype(np.int64) - Jo[bad])
        lev = np.broadcast_to(_LEVEL_OF, Jo.shape)[bad]
        ok = (diff == 1) | ((lev == 1) & (diff == 15))
        assert np.all(ok), "a mismatching code is not the neighbouring cell"
    if enforce_rate:
        assert stats["code_mismatch_rate"] <= CODE_MISMATCH_RATE, stats
    return stats, rg, ro


def check_codes_deep(rec_gpu, rec_oracle, psi, bits):
    """Deep (50-byte) records: psi [n,127] exact oracle angles.  Same rule as check_codes for all 127 codes.
    Returns (stats, radii_gpu [n], radii_oracle [n])."""
    Jg, rg = layout_ref.unpack_canonical_deep(rec_gpu, bits)
    Jo, ro = oracle.unpack_deep(rec_oracle, bits)
    bad = Jg != Jo
    n_bad = int(bad.sum())
    stats = {"angles": int(Jo.size), "code_mismatches": n_bad, "code_mismatch_rate": n_bad / Jo.size}
    if n_bad:
        dist = np.empty_like(psi)
        dist[:, :120] = boundary_distance(psi[:, :120])
        off = 120
        for level, cnt in ((5, 4), (6, 2), (7, 1)):
            _, bnd = oracle.codebook(level, 1 << bits[level - 5])
            a = psi[:, off : off + cnt]
            dist[:, off : off + cnt] = np.min(np.abs(a[..., None] - bnd[1:-1]), axis=-1)
            off += cnt
        worst = float(dist[bad].max())
        stats["worst_mismatch_boundary_distance"] = worst
        assert worst <= ANGLE_TOL, f"code mismatch {worst:.3e} rad away from any boundary"
        diff = np.abs(Jg[bad].astype(np.int64) - Jo[bad])
        lev = np.broadcast_to(np.concatenate([_LEVEL_OF, np.full(7, 5)]), Jo.shape)[bad]
        assert np.all((diff == 1) | ((lev == 1) & (diff == 15))), "a mismatching code is not the neighbouring cell"
    assert stats["code_mismatch_rate"] <= CODE_MISMATCH_RATE, stats
    return stats, rg, ro


def check_radii_deep(rg, ro, y_oracle):
    """rg, ro uint16 [n]: the one radius of each vector; y_oracle [n,128] the oracle's rotated vectors."""
    bad = rg != ro
    n_bad = int(bad.sum())
    stats = {"radii": int(ro.size), "radius_mismatches": n_bad, "radius_mismatch_rate": n_bad / ro.size}
    if n_bad:
        r_exact = np.linalg.norm(y_oracle, axis=1)
        d = np.abs(rg[bad].astype(np.int64) - ro[bad].astype(np.int64))
        assert np.all(d == 1), "radius off by more than one binary16 ulp"
        lo = np.minimum(rg[bad], ro[bad]).astype(np.uint16)
        hi = (lo + 1).astype(np.uint16)
        mid = 0.5 * (lo.view(np.float16).astype(np.float64) + hi.view(np.float16).astype(np.float64))
        rel = np.abs(r_exact[bad] - mid) / mid
        stats["worst_radius_rel_distance"] = float(rel.max())
        assert rel.max() <= RADIUS_REL_TOL, f"radius mismatch {rel.max():.3e} (relative) away from a rounding boundary"
    assert stats["radius_mismatch_rate"] <= RADIUS_MISMATCH_RATE, stats
    return stats


def check_radii(rg, ro, y_oracle, enforce_rate=True):
    """rg, ro uint16 [n,8]; y_oracle [n,128] the oracle's rotated vectors (exact radii)."""
    bad = rg != ro
    n_bad = int(bad.sum())
    stats = {"radii": int(ro.size), "radius_mismatches": n_bad, "radius_mismatch_rate": n_bad / ro.size}
    if n_bad:
        r_exact = np.linalg.norm(y_oracle.reshape(-1, 8, 16), axis=2)
        d = np.abs(rg[bad].astype(np.int64) - ro[bad].astype(np.int64))
        assert np.all(d == 1), "radius off by more than one binary16 ulp"
        # the exact radius must sit next to the rounding boundary between the two candidates
        lo = np.minimum(rg[bad], ro[bad]).astype(np.uint16)
        hi = (lo + 1).astype(np.uint16)
        mid = 0.5 * (lo.view(np.float16).astype(np.float64) + hi.view(np.float16).astype(np.float64))
        rel = np.abs(r_exact[bad] - mid) / mid
        stats["worst_radius_rel_distance"] = float(rel.max())
        assert rel.max() <= RADIUS_REL_TOL, f"radius mismatch {rel.max():.3e} (relative) away from a rounding boundary"
    if enforce_rate:
        assert stats["radius_mismatch_rate"] <= RADIUS_MISMATCH_RATE, stats
    return stats


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def softmax_scale():
    return 1.0 / math.sqrt(128.0)


def upload_records(kind, rec, codes, radii, start, fill=0xFF):
    """Lays canonical records out as tiles (numpy, from the layout specification) and copies them into a device
    cache: rec uint8 [H, n, 62] -> slots [start, start + n) of every head plane; start on a tile boundary.  The rest
    of the last tile gets `fill` in every byte (0xFF: a NaN radius and arbitrary codes)."""
    import torch

    H, n, _ = rec.shape
    assert start % 64 == 0
    T, t0 = (n + 63) // 64, start // 64
    c, r = layout_ref.canonical_to_tiles_planes(kind, rec, T, fill)      # all head planes in one pass
    codes[:, t0:t0 + T] = torch.from_numpy(c).to(codes.device)
    radii[:, t0:t0 + T] = torch.from_numpy(r.view(np.int16)).to(radii.device)


def upload_records_deep(kind, rec, codes, top, start, fill=0xFF):
    """The same for full-depth caches: rec uint8 [H, n, 50]; top: the radius plane, int16 [H, tiles, 128]."""
    import torch

    H, n, _ = rec.shape
    assert start % 64 == 0
    T, t0 = (n + 63) // 64, start // 64
    for h in range(H):
        c, t = layout_ref.canonical_to_tiles_deep(kind, rec[h], T, fill)
        codes[h, t0:t0 + T] = torch.from_numpy(c).to(codes.device)
        top[h, t0:t0 + T] = torch.from_numpy(t.view(np.int16)).to(top.device)
