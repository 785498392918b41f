"""GPU parity of the general format (other bit widths, recursion depths 4..7) against the oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2502_02617_amd import (Context, GeneralFormat, PolarQuantError, general_attn_decode, general_decode,
                                  general_encode, synth)
from tests import helpers, layout_ref

pytestmark = pytest.mark.gpu
DEV = "cuda"
D = 128

FORMATS = [(4, [3, 3, 2, 3]), (4, [4, 3, 3, 3]), (5, [4, 2, 2, 2, 2]), (6, [3, 2, 3, 2, 3, 1]), (7, [4, 3, 2, 2, 1, 2, 3]),
           (4, [4, 2, 2, 2])]


def say(msg):
    print(f"[gpu-test] {msg}", flush=True)


def unpack_general(rec, L, bits):
    """numpy reading of general records -> codes [n, nang], radii bits [n, 128 >> L]"""
    n = rec.shape[0]
    stream = np.unpackbits(rec, axis=1, bitorder="little")
    J, pos = [], 0
    for l in range(1, L + 1):
        w, cnt = bits[l - 1], D >> l
        field = stream[:, pos:pos + cnt * w].reshape(n, cnt, w).astype(np.int32)
        J.append((field << np.arange(w)).sum(axis=2))
        pos += cnt * w
    code_bytes = (pos + 7) // 8
    return np.concatenate(J, axis=1), rec[:, code_bytes:].copy().view(np.uint16)


def level_boundaries(cbg, L, bits):
    out, off = [], 0
    for l in range(1, L + 1):
        K = 1 << bits[l - 1]
        c = cbg[off:off + K]
        out.append(0.5 * (c[1:] + c[:-1]))
        off += K
    return out


@pytest.mark.parametrize("L,bits", FORMATS)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_general_format_encode_decode(L, bits, dtype):
    say(f"general format depth {L} bits {bits} {dtype}: encode, DeQuant")
    ctx = Context(seed=11)
    S = ctx.preconditioner()
    fmt = GeneralFormat(L, bits)
    cbg_lib = fmt.codebooks()
    cbg = oracle.general_codebooks(L, bits)
    assert np.max(np.abs(cbg_lib - cbg)) < 1e-12          # two integrators, one fixed point
    rb = fmt.record_bytes()
    assert rb == oracle.general_record_bytes(L, bits)
    n = 3000
    if dtype == torch.bfloat16:
        x = synth.kv_stream(n, 1, seed=40 + L).reshape(n, D)
    else:
        x = synth.gaussian_vectors(n, seed=41 + L)
    rec_gpu = torch.full((n, rb), 0xA5, dtype=torch.uint8, device=DEV)
    general_encode(ctx, fmt, cbg, x.to(DEV), rec_gpu)
    torch.cuda.synchronize()
    rec_or, psi, J_or = oracle.encode_general(x.double().numpy(), S, L, bits, cbg, want_psi=True, want_codes=True)
    J_gpu, r_gpu = unpack_general(rec_gpu.cpu().numpy(), L, bits)
    r_or = rec_or[:, -2 * (D >> L):].copy().view(np.uint16)
    # codes: bit-exact except where the oracle's exact angle is within 1e-5 rad of a cell boundary (neighbouring cell)
    bad = J_gpu != J_or
    off, worst = 0, 0.0
    for l, bnd in enumerate(level_boundaries(cbg, L, bits), start=1):
        cnt = D >> l
        sub = bad[:, off:off + cnt]
        if sub.any():
            ang = psi[:, off:off + cnt][sub]
            dist = np.min(np.abs(ang[:, None] - bnd[None, :]), axis=1)
            assert np.all(np.abs(J_gpu[:, off:off + cnt][sub] - J_or[:, off:off + cnt][sub]) == 1)
            worst = max(worst, float(dist.max()))
        off += cnt
    assert worst <= 1e-5 and bad.mean() <= 1e-4
    # radii: binary16 bits equal, or one step apart where the exact radius sits on a rounding boundary
    y = x.double().numpy() @ S
    exact = np.linalg.norm(y.reshape(n, D >> L, -1), axis=2)
    diff = r_gpu.astype(np.int32) - r_or.astype(np.int32)
    assert np.all(np.abs(diff) <= 1)
    if (diff != 0).any():
        lo = np.minimum(r_gpu, r_or)[diff != 0].view(np.float16).astype(np.float64)
        hi = np.maximum(r_gpu, r_or)[diff != 0].view(np.float16).astype(np.float64)
        assert np.all(np.abs(exact[diff != 0] - 0.5 * (lo + hi)) <= 1e-6 * exact[diff != 0])
    assert (diff != 0).mean() <= 2e-3
    say(f"  {bad.sum()} code mismatches of {bad.size} (worst boundary distance {worst:.1e}), {(diff != 0).sum()} radius ties of {diff.size}")
    # DeQuant of the oracle's records: with and without the trailing S^T
    rec_dev = torch.from_numpy(rec_or).to(DEV)
    out = torch.empty((n, D), dtype=torch.float32, device=DEV)
    for rotated in (False, True):
        general_decode(ctx, fmt, cbg, rec_dev, n, out, rotated=rotated)
        torch.cuda.synchronize()
        ref = oracle.decode_general(rec_or, S, L, bits, cbg, rotated=rotated)
        err = helpers.rel_l2(out.cpu().numpy().astype(np.float64), ref)
        say(f"  DeQuant rotated={rotated}: rel L2 {err:.2e}")
        assert err <= 1e-5


@pytest.mark.parametrize("L,bits", FORMATS)
def test_general_format_attention(L, bits):
    say(f"general format depth {L} bits {bits}: attention")
    ctx = Context(seed=12)
    S = ctx.preconditioner()
    fmt = GeneralFormat(L, bits)
    cbg = oracle.general_codebooks(L, bits)
    rb = fmt.record_bytes()
    Hkv, Hq = 2, 8
    lens = [1, 70, 0, 333, 129]
    starts, pool = [], 0
    for nt in lens:
        starts.append(pool)
        pool += max(nt, 1) + 3            # no alignment is asked of the general layout
    k_rec = np.full((Hkv, pool, rb), 0xFF, dtype=np.uint8)
    v_rec = np.full((Hkv, pool, rb), 0xFF, dtype=np.uint8)
    for b, nt in enumerate(lens):
        if nt == 0:
            continue
        k = synth.kv_stream(nt, Hkv, seed=500 + 2 * b).double().numpy()       # [Hkv, nt, 128]
        v = synth.kv_stream(nt, Hkv, seed=501 + 2 * b).double().numpy()
        for h in range(Hkv):
            k_rec[h, starts[b]:starts[b] + nt] = oracle.encode_general(k[h], S, L, bits, cbg)
            v_rec[h, starts[b]:starts[b] + nt] = oracle.encode_general(v[h], S, L, bits, cbg)
    q = synth.queries(len(lens), Hq, seed=77)
    out = torch.full((len(lens), Hq, D), float("nan"), dtype=torch.float32, device=DEV)
    st = torch.tensor(starts, dtype=torch.int64, device=DEV)
    cl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    general_attn_decode(ctx, fmt, cbg, q.to(DEV), out, torch.from_numpy(k_rec).to(DEV), torch.from_numpy(v_rec).to(DEV),
                        st, cl, helpers.softmax_scale())
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.attention_general(q.double().numpy(), k_rec, v_rec, np.array(starts), np.array(lens, np.int32), S, L, bits,
                                   cbg, helpers.softmax_scale())
    assert np.all(np.isfinite(got)) and np.all(got[2] == 0.0)
    err = helpers.rel_l2(got, ref)
    say(f"  rel L2 {err:.2e}")
    assert err <= 2e-3


def test_general_format_with_section_4_1_settings_matches_the_tuned_path():
    """Depth 4, bits 4/2/2/2 through the general kernels: the same codes and radii as the tuned encoder's records."""
    say("general format at Section 4.1's settings against the tuned encoder")
    ctx = Context(seed=13)
    fmt = GeneralFormat(4, [4, 2, 2, 2])
    cbg = fmt.codebooks()
    n = 2048
    x = synth.kv_stream(n, 1, seed=90)                        # [1, n, 128] bf16
    rec_g = torch.empty((n, fmt.record_bytes()), dtype=torch.uint8, device=DEV)
    general_encode(ctx, fmt, cbg, x.reshape(n, D).to(DEV), rec_g)
    codes, radii = Context.alloc_cache(1, n, DEV)
    ctx.encode_kv(x.permute(1, 0, 2).contiguous().to(DEV), 0, codes, radii)
    rec_t = torch.empty((1, n, 62), dtype=torch.uint8, device=DEV)
    ctx.export_canonical(0, codes, radii, 0, n, rec_t)
    torch.cuda.synchronize()
    J_g, r_g = unpack_general(rec_g.cpu().numpy(), 4, [4, 2, 2, 2])
    J_t, r_t = layout_ref.unpack_canonical(rec_t.cpu().numpy().reshape(n, 62))   # numpy reader of the canonical record
    assert (J_g != J_t).mean() <= 1e-4 and np.all(np.abs(r_g.astype(np.int32) - r_t.astype(np.int32)) <= 1)


def test_general_format_refuses_what_it_does_not_cover():
    for L, bits in [(3, [4, 2, 2]), (8, [4, 2, 2, 2, 2, 2, 2]), (4, [5, 2, 2, 2]), (4, [4, 1, 2, 2]), (5, [4, 2, 2, 2, 4])]:
        with pytest.raises(PolarQuantError):
            GeneralFormat(L, bits).record_bytes()
