"""GPU parity: libpolarquant's HIP kernels against the fp64 oracle, through the C ABI.

Every input is seeded and synthetic (see paper_2502_02617_amd/synth.py).  Each test
prints what it is about to run before touching the GPU.
"""
import math
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2502_02617_amd import Context, PQ_KEY, PQ_VALUE, PolarQuantError, synth
from tests import helpers, layout_ref

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def env():
    ctx = Context(seed=0)
    S = oracle.preconditioner(0)
    cb = oracle.default_codebooks()
    return ctx, S, cb


def gpu_encode(ctx, x_cpu, kind, pool_tokens, dst0=0, prefill=None):
    """x_cpu [T, H, 128] -> (codes, radii) device tensors after pq_encode_kv."""
    T, H, _ = x_cpu.shape
    codes, radii = Context.alloc_cache(H, pool_tokens, DEV)
    if prefill is None:
        codes.fill_(0xA5)  # stale bytes must never leak into written slots
        radii.fill_(0x5A5A)
    else:
        codes.copy_(prefill[0])
        radii.copy_(prefill[1])
    x = x_cpu.to(DEV)
    ctx.encode_kv(x, kind, codes, radii, dst_token0=dst0)
    torch.cuda.synchronize()
    return codes, radii


def canonical_both_ways(ctx, kind, codes, radii, token0, n_tokens):
    """Records via the library's export kernel and via the independent numpy reading of the layout."""
    H = codes.shape[0]
    rec = torch.empty((H, n_tokens, 62), dtype=torch.uint8, device=DEV)
    ctx.export_canonical(kind, codes, radii, token0, n_tokens, rec)
    torch.cuda.synchronize()
    rec_lib = rec.cpu().numpy()
    c = codes.cpu().numpy()
    r = radii.cpu().numpy().view(np.uint16)
    assert token0 % 64 == 0
    t0 = token0 // 64
    rec_np = np.stack([layout_ref.tiles_to_canonical(kind, c[h, t0:], r[h, t0:], n_tokens) for h in range(H)])
    assert np.array_equal(rec_lib, rec_np), "export kernel and layout specification disagree"
    return rec_lib


def oracle_records(x_cpu, S, cb):
    """x_cpu [T, H, 128] -> records [H, T, 62], psi [H, T, 120], y [H, T, 128]."""
    T, H, _ = x_cpu.shape
    xs = x_cpu.permute(1, 0, 2).contiguous().to(torch.float64).numpy().reshape(H * T, 128)
    rec, psi, y = oracle.encode(xs, S, cb, want_psi=True, want_y=True)
    return rec.reshape(H, T, 62), psi.reshape(H, T, 120), y.reshape(H, T, 128)


def check_encode(ctx, S, cb, x_cpu, kind, label):
    T, H, _ = x_cpu.shape
    pool = ((T + 63) // 64) * 64
    say(f"encode parity {label}: T={T} H={H} kind={kind} dtype={x_cpu.dtype}")
    codes, radii = gpu_encode(ctx, x_cpu, kind, pool)
    rec_gpu = canonical_both_ways(ctx, kind, codes, radii, 0, T)
    rec_or, psi, y = oracle_records(x_cpu, S, cb)
    st, rg, ro = helpers.check_codes(rec_gpu.reshape(-1, 62), rec_or.reshape(-1, 62), psi.reshape(-1, 120), cb=cb)
    st.update(helpers.check_radii(rg, ro, y.reshape(-1, 128)))
    say(f"  {st}")
    return codes, radii, rec_gpu, rec_or


# ---------------------------------------------------------------------------
# config 0: 1024 fp32 N(0,1) vectors, round trip
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kind", [PQ_KEY, PQ_VALUE])
def test_config0_round_trip(env, kind):
    ctx, S, cb = env
    x = synth.gaussian_vectors(1024, seed=0).reshape(1024, 1, 128)
    codes, radii, rec_gpu, rec_or = check_encode(ctx, S, cb, x, kind, "config 0")
    # DeQuant on identical codes: the oracle's records laid out as tiles, which isolates the decode arithmetic;
    # and DeQuant of the library's own cache against the oracle end to end
    codes_or, radii_or = Context.alloc_cache(1, 1024, DEV)
    helpers.upload_records(kind, rec_or, codes_or, radii_or, 0)
    out = torch.empty((1024, 1, 128), dtype=torch.float32, device=DEV)
    out_or = torch.empty_like(out)
    for rotated in (True, False):
        ctx.decode_kv(kind, codes, radii, 0, 1024, out, rotated=rotated)
        ctx.decode_kv(kind, codes_or, radii_or, 0, 1024, out_or, rotated=rotated)
        torch.cuda.synchronize()
        ref_or = oracle.decode(rec_or[0], S, cb, rotated=rotated)
        e_same = helpers.rel_l2(out_or.cpu().numpy()[:, 0], ref_or)
        e_or = helpers.rel_l2(out.cpu().numpy()[:, 0], ref_or)
        say(f"  decode rotated={rotated}: rel L2 vs oracle on same codes {e_same:.2e}, end to end {e_or:.2e}")
        assert e_same <= 1e-5 and e_or <= 1e-3
    # reconstruction error of the scheme itself (regression value pinned in the CPU tests)
    rel = helpers.rel_l2(out.cpu().numpy()[:, 0], x[:, 0].numpy())
    assert 0.17 < rel < 0.19
    # bf16 output path
    outb = torch.empty((1024, 1, 128), dtype=torch.bfloat16, device=DEV)
    ctx.decode_kv(kind, codes, radii, 0, 1024, outb, rotated=False)
    torch.cuda.synchronize()
    assert helpers.rel_l2(outb.float().cpu().numpy()[:, 0], out.cpu().numpy()[:, 0]) <= 4e-3


# ---------------------------------------------------------------------------
# config 1 shape at reduced length: bf16 with outlier channels, ragged tail
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kind", [PQ_KEY, PQ_VALUE])
def test_encode_bf16_outliers_ragged_tail(env, kind):
    ctx, S, cb = env
    T = 64 * 9 + 37  # several tiles and a ragged tail
    x = synth.kv_stream(T, 8, seed=1).permute(1, 0, 2).contiguous()  # [T, 8, 128] bf16
    check_encode(ctx, S, cb, x, kind, "config 1 (reduced)")


def test_encode_strided_input_and_offsets(env):
    ctx, S, cb = env
    # head-major source [H, T, 128] read through strides; destination starts mid-tile
    H, T, dst0, pool = 3, 150, 100, 320
    src = synth.kv_stream(T, H, seed=5)  # [H, T, 128]
    for kind in (PQ_KEY, PQ_VALUE):
        say(f"strided encode kind={kind}")
        codes, radii = Context.alloc_cache(H, pool, DEV)
        codes.zero_()
        radii.zero_()
        # slots [0, 100) written first by another call, must survive the second one
        first = synth.kv_stream(dst0, H, seed=6).permute(1, 0, 2).contiguous()
        ctx.encode_kv(first.to(DEV), kind, codes, radii, dst_token0=0)
        xs = src.to(DEV)
        ctx.encode_kv(xs, kind, codes, radii, dst_token0=dst0, ld_token=xs.stride(1), ld_head=xs.stride(0),
                      n_tokens=T, n_heads=H)
        torch.cuda.synchronize()
        rec = canonical_both_ways(ctx, kind, codes, radii, 0, dst0 + T)
        both = torch.cat([first, src.permute(1, 0, 2)], dim=0)
        rec_or, psi, y = oracle_records(both, S, cb)
        st, rg, ro = helpers.check_codes(rec.reshape(-1, 62), rec_or.reshape(-1, 62), psi.reshape(-1, 120))
        helpers.check_radii(rg, ro, y.reshape(-1, 128))


def test_append_one_token_per_sequence(env):
    run_append_case(*env)


def run_append_case(ctx, S, cb):
    H, pool = 2, 64 * 6
    lens = [0, 63, 64, 100]           # tokens already cached per sequence
    starts = [0, 64, 128, 256]        # tile-aligned sequence starts
    for kind in (PQ_KEY, PQ_VALUE):
        say(f"append kind={kind}")
        codes, radii = Context.alloc_cache(H, pool, DEV)
        codes.zero_()
        radii.zero_()
        hist = []
        for b, (s0, n) in enumerate(zip(starts, lens)):
            xb = synth.kv_stream(max(n, 1), H, seed=40 + b).permute(1, 0, 2).contiguous()[:n]
            hist.append(xb)
            if n:
                ctx.encode_kv(xb.to(DEV), kind, codes, radii, dst_token0=s0)
        new = synth.kv_stream(len(lens), H, seed=50).permute(1, 0, 2).contiguous()  # [B, H, 128]
        dst = torch.tensor([s0 + n for s0, n in zip(starts, lens)], dtype=torch.int64, device=DEV)
        ctx.append_kv(new.to(DEV), kind, codes, radii, dst)
        torch.cuda.synchronize()
        for b, (s0, n) in enumerate(zip(starts, lens)):
            full = torch.cat([hist[b], new[b : b + 1]], dim=0)
            rec = canonical_both_ways(ctx, kind, codes, radii, s0, n + 1)
            rec_or, psi, y = oracle_records(full, S, cb)
            st, rg, ro = helpers.check_codes(rec.reshape(-1, 62), rec_or.reshape(-1, 62), psi.reshape(-1, 120))
            helpers.check_radii(rg, ro, y.reshape(-1, 128))


def test_append_pair_equals_two_appends(env):
    """pq_append_kv_pair writes what pq_append_kv(keys) + pq_append_kv(values) write, bit for bit."""
    ctx, S, cb = env
    say("append pair vs two single appends")
    H, B, pool = 3, 5, 64 * 5
    dst = torch.tensor([0, 64 + 63, 128 + 1, 192 + 30, 256 + 17], dtype=torch.int64, device=DEV)
    caches = []
    for _ in range(2):
        kc, kr = Context.alloc_cache(H, pool, DEV)
        vc, vr = Context.alloc_cache(H, pool, DEV)
        old_k = synth.kv_stream(pool, H, seed=60).permute(1, 0, 2).contiguous().to(DEV)
        old_v = synth.kv_stream(pool, H, seed=61).permute(1, 0, 2).contiguous().to(DEV)
        ctx.encode_kv(old_k, PQ_KEY, kc, kr)      # neighbours of the patched slots must survive
        ctx.encode_kv(old_v, PQ_VALUE, vc, vr)
        caches.append((kc, kr, vc, vr))
    for dtype in (torch.bfloat16, torch.float32):
        nk = synth.kv_stream(B, H, seed=62).permute(1, 0, 2).contiguous().to(dtype).to(DEV)
        nv = synth.kv_stream(B, H, seed=63).permute(1, 0, 2).contiguous().to(dtype).to(DEV)
        kc, kr, vc, vr = caches[0]
        ctx.append_kv(nk, PQ_KEY, kc, kr, dst)
        ctx.append_kv(nv, PQ_VALUE, vc, vr, dst)
        kc2, kr2, vc2, vr2 = caches[1]
        ctx.append_kv_pair(nk, nv, kc2, kr2, vc2, vr2, dst)
        torch.cuda.synchronize()
        for a, b in zip(caches[0], caches[1]):
            assert torch.equal(a, b)
    # and against the oracle on the patched slots
    kc2, kr2, vc2, vr2 = caches[1]
    for kind, codes, radii, x in ((PQ_KEY, kc2, kr2, nk), (PQ_VALUE, vc2, vr2, nv)):
        for b in range(B):
            slot = int(dst[b])
            rec = canonical_both_ways(ctx, kind, codes, radii, slot - slot % 64, 64)[:, slot % 64]
            rec_or, psi, y = oracle_records(x[b:b + 1].cpu(), S, cb)
            st, rg, ro = helpers.check_codes(rec.reshape(-1, 62), rec_or.reshape(-1, 62), psi.reshape(-1, 120))
            helpers.check_radii(rg, ro, y.reshape(-1, 128))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_encode_pair_equals_two_encodes(env, dtype):
    """pq_encode_kv_pair writes exactly what the two single-stream calls write: full tiles, partial tiles at
    both ends of the range, several heads, a strided view as input."""
    ctx, S, cb = env
    T, H, pool, dst0 = 64 * 5 + 23, 3, 64 * 8, 37
    say(f"encode pair vs two encodes: T={T} H={H} dtype={dtype} dst0={dst0}")
    if dtype == torch.bfloat16:
        xk = synth.kv_stream(T, H, seed=310).permute(1, 0, 2).contiguous()
        xv = synth.kv_stream(T, H, seed=311).permute(1, 0, 2).contiguous()
    else:
        xk = synth.gaussian_vectors(T * H, seed=312).reshape(T, H, 128)
        xv = synth.gaussian_vectors(T * H, seed=313).reshape(T, H, 128)
    xk, xv = xk.to(DEV), xv.to(DEV)
    ref = []
    for kind, x in ((PQ_KEY, xk), (PQ_VALUE, xv)):
        codes, radii = Context.alloc_cache(H, pool, DEV)
        codes.fill_(0x3C)
        radii.fill_(0x1234)
        ctx.encode_kv(x, kind, codes, radii, dst_token0=dst0)
        ref.append((codes, radii))
    kc, kr = Context.alloc_cache(H, pool, DEV)
    vc, vr = Context.alloc_cache(H, pool, DEV)
    for t in (kc, vc):
        t.fill_(0x3C)
    for t in (kr, vr):
        t.fill_(0x1234)
    ctx.encode_kv_pair(xk, xv, kc, kr, vc, vr, dst_token0=dst0)
    torch.cuda.synchronize()
    assert torch.equal(kc, ref[0][0]) and torch.equal(kr, ref[0][1])
    assert torch.equal(vc, ref[1][0]) and torch.equal(vr, ref[1][1])
    # and the records are the oracle's (keys; the single-stream call is checked against it elsewhere too)
    rec = canonical_both_ways(ctx, PQ_KEY, kc, kr, 0, 64 * 6)[:, dst0:dst0 + T]
    rec_or, psi, y = oracle_records(xk.cpu(), S, cb)
    st, rg, ro = helpers.check_codes(rec.reshape(-1, 62), rec_or.reshape(-1, 62), psi.reshape(-1, 120))
    helpers.check_radii(rg, ro, y.reshape(-1, 128))


def test_encode_degenerate_inputs(env):
    ctx, S, cb = env
    say("degenerate encode inputs")
    x = torch.zeros((70, 1, 128), dtype=torch.bfloat16)
    x[1, 0, 5] = 1.0          # a single non-zero coordinate
    x[2, 0, :] = -3.0         # constant vector
    x[3, 0, 0] = 2.0 ** -20   # tiny
    x[4, 0, :] = 200.0        # large but inside binary16 range after rotation
    for kind in (PQ_KEY, PQ_VALUE):
        codes, radii = gpu_encode(ctx, x, kind, 128)
        rec = canonical_both_ways(ctx, kind, codes, radii, 0, 70)
        rec_or, psi, y = oracle_records(x, S, cb)
        J, r = layout_ref.unpack_canonical(rec[0])
        assert np.all(J[0] == 0) and np.all(r[0] == 0)  # zero vector -> all-zero record
        st, rg, ro = helpers.check_codes(rec.reshape(-1, 62), rec_or.reshape(-1, 62), psi.reshape(-1, 120))
        helpers.check_radii(rg, ro, y.reshape(-1, 128))
    # n_tokens == 0 is a no-op
    codes, radii = Context.alloc_cache(1, 64, DEV)
    ctx.encode_kv(torch.zeros((0, 1, 128), dtype=torch.bfloat16, device=DEV), PQ_KEY, codes, radii)
    with pytest.raises(PolarQuantError):
        ctx.encode_kv(torch.zeros((65, 1, 128), dtype=torch.bfloat16, device=DEV), PQ_KEY, codes, radii)


def test_extreme_block_norms(env):
    """Block norms beyond the binary16 range: the stored radius saturates at 65504 (0x7BFF) in the library exactly as
    in the oracle (Section 4.1 fixes 16-bit radii and is silent beyond their range), codes are unaffected, and
    attention on such records stays finite and within the usual bound."""
    ctx, S, cb = env
    say("extreme block norms: radii saturate at the largest finite binary16")
    g = torch.Generator().manual_seed(77)
    n, H = 130, 2
    x = torch.randn((n, H, 128), generator=g, dtype=torch.float32)
    x[0::3] *= 3.0e4                      # every block of these vectors has a norm far beyond 65504
    x[1::3, :, 32:48] *= 1.0e5            # one block beyond the range, the others ordinary
    for kind in (PQ_KEY, PQ_VALUE):
        codes, radii = gpu_encode(ctx, x, kind, 192)
        rec = canonical_both_ways(ctx, kind, codes, radii, 0, n)
        rec_or, psi, y = oracle_records(x, S, cb)
        st, rg, ro = helpers.check_codes(rec.reshape(-1, 62), rec_or.reshape(-1, 62), psi.reshape(-1, 120))
        helpers.check_radii(rg, ro, y.reshape(-1, 128))
        sat = ro == 0x7BFF
        assert sat.sum() >= (n // 3) * H * 8 and np.array_equal(rg[sat], ro[sat])
        assert not np.any((rg & 0x7C00) == 0x7C00)  # no infinity, no NaN
    # attention on the oracle's records of such vectors: huge values under ordinary keys, and huge keys
    lens = [n, n]
    rec_x = oracle_records(x, S, cb)[0]
    rec_n = oracle_records(torch.randn((n, H, 128), generator=g, dtype=torch.float32), S, cb)[0]
    pool = 2 * 192
    kc, kr = Context.alloc_cache(H, pool, DEV)
    vc, vr = Context.alloc_cache(H, pool, DEV)
    k_rec = np.zeros((H, pool, 62), dtype=np.uint8)
    v_rec = np.zeros((H, pool, 62), dtype=np.uint8)
    for b, (rk, rv) in enumerate(((rec_n, rec_x), (rec_x, rec_n))):
        k_rec[:, 192 * b : 192 * b + n] = rk
        v_rec[:, 192 * b : 192 * b + n] = rv
        helpers.upload_records(PQ_KEY, rk, kc, kr, 192 * b)
        helpers.upload_records(PQ_VALUE, rv, vc, vr, 192 * b)
    starts = np.array([0, 192], dtype=np.int64)
    q = synth.queries(2, 4, seed=78)
    got = gpu_attention(ctx, q, (kc, kr, vc, vr), starts, lens)
    ref = oracle.attention(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb,
                           helpers.softmax_scale())
    assert np.all(np.isfinite(got))
    errs = [helpers.rel_l2(got[b], ref[b]) for b in range(2)]
    say(f"  attention rel L2: huge values {errs[0]:.2e}, huge keys {errs[1]:.2e}")
    assert max(errs) <= 2e-3


# ---------------------------------------------------------------------------
# attention
# ---------------------------------------------------------------------------
def build_cache(ctx, S, cb, lens, Hkv, seed, want_oracle=True):
    """Ragged batch: returns device caches, seq_start, and oracle records [Hkv, pool, 62].
    The attention kernels are tested on the oracle's own records, laid out as tiles by the numpy layout reference
    and copied to the device: both sides then work on identical codes and radii, and nothing that a library kernel
    produced reaches the oracle.  (The encoder has its own parity tests; an angle within 1e-5 rad of a cell boundary
    may legitimately be coded either way there, and a tie in one heavily weighted token would otherwise show up as
    an attention error.)  want_oracle=False: the cache is filled by the library's encoder and no records are made."""
    B = len(lens)
    starts, pool = [], 0
    for n in lens:
        starts.append(pool)
        pool += ((max(n, 1) + 63) // 64) * 64
    kc, kr = Context.alloc_cache(Hkv, pool, DEV)
    vc, vr = Context.alloc_cache(Hkv, pool, DEV)
    for t in (kc, vc):
        t.fill_(0xFF)      # stale slots hold NaN-like garbage on purpose
    for t in (kr, vr):
        t.fill_(0x7E00)    # binary16 NaN
    k_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
    v_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
    for b, n in enumerate(lens):
        if n == 0:
            continue
        k = synth.kv_stream(n, Hkv, seed + 2 * b).permute(1, 0, 2).contiguous()
        v = synth.kv_stream(n, Hkv, seed + 2 * b + 1).permute(1, 0, 2).contiguous()
        if want_oracle:
            for kind, x, codes, radii, rec in ((PQ_KEY, k, kc, kr, k_rec), (PQ_VALUE, v, vc, vr, v_rec)):
                rec_or = oracle_records(x, S, cb)[0]
                rec[:, starts[b] : starts[b] + n] = rec_or
                helpers.upload_records(kind, rec_or, codes, radii, starts[b])
        else:
            ctx.encode_kv(k.to(DEV), PQ_KEY, kc, kr, dst_token0=starts[b])
            ctx.encode_kv(v.to(DEV), PQ_VALUE, vc, vr, dst_token0=starts[b])
    torch.cuda.synchronize()
    return (kc, kr, vc, vr), np.array(starts, dtype=np.int64), pool, k_rec, v_rec


def gpu_attention(ctx, q_cpu, caches, starts, lens, max_ctx=None, out_dtype=torch.float32):
    B, Hq, _ = q_cpu.shape
    kc, kr, vc, vr = caches
    Hkv = kc.shape[0]
    max_ctx = max(max(lens), 1) if max_ctx is None else max_ctx
    ws = torch.empty(Context.attn_workspace_bytes(B, Hq, Hkv, max_ctx), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    out = torch.full((B, Hq, 128), float("nan"), dtype=out_dtype, device=DEV)
    ctx.attn_decode_polar(q_cpu.to(DEV), out, kc, kr, vc, vr,
                          torch.from_numpy(starts).to(DEV), torch.tensor(lens, dtype=torch.int32, device=DEV),
                          max_ctx, helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy()


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (4, 2), (3, 3), (6, 2), (5, 1), (12, 2), (14, 2), (16, 1)])
def test_attention_small_ragged(env, Hq, Hkv):
    ctx, S, cb = env
    lens = [1, 17, 64, 65, 200, 0, 700, 1030]
    say(f"attention small ragged Hq={Hq} Hkv={Hkv} lens={lens}")
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, Hkv, seed=100)
    q = synth.queries(len(lens), Hq, seed=100)
    got = gpu_attention(ctx, q, caches, starts, lens)
    ref = oracle.attention(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb,
                           helpers.softmax_scale())
    assert np.all(np.isfinite(got))
    assert np.all(got[5] == 0.0)  # empty context -> zero row
    err = helpers.rel_l2(got, ref)
    rows = [helpers.rel_l2(got[b], ref[b]) for b in range(len(lens)) if lens[b]]
    say(f"  rel L2 all rows {err:.2e}; per sequence {['%.1e' % r for r in rows]}")
    assert err <= 2e-3
    assert max(rows) <= 4e-3
    # bf16 output: the same numbers rounded to nearest even; against the oracle the format's own
    # rounding error (about 2^-9 relative per element) comes on top of the 2e-3 budget
    got_bf = gpu_attention(ctx, q, caches, starts, lens, out_dtype=torch.bfloat16)
    assert np.array_equal(got_bf, torch.from_numpy(got).to(torch.bfloat16).float().numpy())
    fmt = helpers.rel_l2(torch.from_numpy(ref).to(torch.bfloat16).double().numpy(), ref)
    assert helpers.rel_l2(got_bf, ref) <= math.sqrt(2e-3 ** 2 + fmt ** 2)
    # a larger max_ctx than needed (another launch shape) gives the same answer up to reduction order
    got2 = gpu_attention(ctx, q, caches, starts, lens, max_ctx=pool)
    assert helpers.rel_l2(got2, ref) <= 2e-3


def test_attention_is_deterministic_and_split_invariant(env):
    ctx, S, cb = env
    lens = [5000, 3000]
    say(f"attention determinism lens={lens}")
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, 2, seed=300, want_oracle=False)
    q = synth.queries(2, 8, seed=300)
    a = gpu_attention(ctx, q, caches, starts, lens)
    b = gpu_attention(ctx, q, caches, starts, lens)
    assert np.array_equal(a, b)  # fixed-order combine: run-to-run identical
    c = gpu_attention(ctx, q, caches, starts, lens, max_ctx=pool)  # different chunking
    assert helpers.rel_l2(c, a) <= 2e-3


def test_two_streams_with_one_context_do_not_interfere(env):
    """One context, two HIP streams (default priority), each with its own workspace, cache and output: decode steps
    issued alternately on both streams give, bit for bit, what each gives alone -- the library keeps no mutable
    state between calls besides what the caller passes in."""
    ctx, S, cb = env
    say("two streams, one context")
    Hq, Hkv = 8, 2
    jobs = []
    for j, lens in enumerate(([3000, 65, 700], [1200, 2500])):
        caches, starts, pool, _, _ = build_cache(ctx, S, cb, lens, Hkv, seed=360 + 10 * j, want_oracle=False)
        B = len(lens)
        q = synth.queries(B, Hq, seed=361 + j).to(DEV)
        nk = synth.kv_stream(B, Hkv, 362 + j).permute(1, 0, 2).contiguous().to(DEV)
        nv = synth.kv_stream(B, Hkv, 364 + j).permute(1, 0, 2).contiguous().to(DEV)
        seq_start = torch.from_numpy(starts).to(DEV)
        ctx_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
        dst = seq_start + ctx_len.to(torch.int64) - 1          # the step overwrites the newest slot
        ws = torch.empty(Context.attn_workspace_bytes(B, Hq, Hkv, max(lens)), dtype=torch.uint8, device=DEV)
        out = torch.empty((B, Hq, 128), dtype=torch.float32, device=DEV)
        jobs.append(dict(caches=caches, q=q, nk=nk, nv=nv, seq_start=seq_start, ctx_len=ctx_len, dst=dst, ws=ws, out=out,
                         max_ctx=max(lens)))

    def step(job):
        kc, kr, vc, vr = job["caches"]
        ctx.decode_step_polar(job["nk"], job["nv"], job["dst"], job["q"], job["out"], kc, kr, vc, vr, job["seq_start"],
                              job["ctx_len"], job["max_ctx"], helpers.softmax_scale(), job["ws"])

    alone = []
    for job in jobs:
        step(job)
        torch.cuda.synchronize()
        alone.append(job["out"].clone())
        job["out"].fill_(float("nan"))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for _ in range(20):
        for job, st in zip(jobs, streams):
            with torch.cuda.stream(st):
                step(job)
    torch.cuda.synchronize()
    for job, ref in zip(jobs, alone):
        assert torch.equal(job["out"], ref)


def test_attention_medium_against_oracle(env):
    ctx, S, cb = env
    lens = [4096 + 13, 2500]
    say(f"attention medium lens={lens}")
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, 8, seed=500)
    q = synth.queries(2, 32, seed=500)
    got = gpu_attention(ctx, q, caches, starts, lens)
    ref = oracle.attention(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb,
                           helpers.softmax_scale())
    err = helpers.rel_l2(got, ref)
    say(f"  rel L2 {err:.2e}")
    assert err <= 2e-3


@pytest.mark.parametrize("B,Hq,Hkv,lo,hi", [(70, 8, 2, 1, 400), (130, 4, 1, 1, 150), (70, 32, 8, 1500, 2500),
                                            (600, 2, 1, 1, 70)])
def test_attention_many_sequences(env, B, Hq, Hkv, lo, hi):
    """More than 64 sequences (the per-sequence table of the work plan is then read from global
    memory instead of LDS), empty sequences in between, and wavefront shares that run across
    the boundaries of several (sequence, kv head) streams.  600 sequences: the running sum of the
    plan takes more than one round of 512."""
    ctx, S, cb = env
    rng = np.random.default_rng(B * 1000 + hi)
    lens = [int(n) for n in rng.integers(lo, hi + 1, size=B)]
    for b in (0, 7, 8, 40, B - 1):  # empty sequences: the first, two neighbours, one in the middle, the last
        lens[b] = 0
    say(f"attention, {B} sequences, Hq={Hq} Hkv={Hkv}, lengths {lo}..{hi}, {sum(lens)} tokens")
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, Hkv, seed=7000 + B)
    q = synth.queries(B, Hq, seed=7000 + B)
    got = gpu_attention(ctx, q, caches, starts, lens)
    ref = oracle.attention(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb,
                           helpers.softmax_scale())
    assert np.all(np.isfinite(got))
    for b in range(B):
        if lens[b] == 0:
            assert np.all(got[b] == 0.0)
    err = helpers.rel_l2(got, ref)
    rows = [helpers.rel_l2(got[b], ref[b]) for b in range(B) if lens[b]]
    say(f"  rel L2 all rows {err:.2e}; worst sequence {max(rows):.2e}")
    assert err <= 2e-3
    assert max(rows) <= 4e-3
    # a larger max_ctx (another launch size, possibly another split) gives the same answer up to reduction order
    got2 = gpu_attention(ctx, q, caches, starts, lens, max_ctx=pool)
    assert helpers.rel_l2(got2, ref) <= 2e-3


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5, 6])
def test_attention_random_batch_shapes(env, seed):
    """Batch size, head counts and context lengths drawn at random (seeded): the device-side split of the
    work has to cover every tile of every stream exactly once whatever the mix."""
    ctx, S, cb = env
    rng = np.random.default_rng(9000 + seed)
    B = int(rng.integers(1, 100))
    Hkv = int(rng.choice([1, 2, 3, 8]))
    G = int(rng.choice([1, 2, 4, 8]))
    Hq = Hkv * G
    hi = int(rng.choice([3, 70, 300, 900]))
    lens = [int(n) for n in rng.integers(0, hi + 1, size=B)]
    if sum(lens) == 0:
        lens[0] = 1
    say(f"attention, random shapes seed {seed}: B={B} Hq={Hq} Hkv={Hkv} lengths 0..{hi}, {sum(lens)} tokens")
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, Hkv, seed=9100 + 10 * seed)
    q = synth.queries(B, Hq, seed=9200 + seed)
    got = gpu_attention(ctx, q, caches, starts, lens)
    ref = oracle.attention(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb,
                           helpers.softmax_scale())
    assert np.all(np.isfinite(got))
    for b in range(B):
        if lens[b] == 0:
            assert np.all(got[b] == 0.0)
    err = helpers.rel_l2(got, ref)
    say(f"  rel L2 all rows {err:.2e}")
    assert err <= 2e-3


@pytest.mark.parametrize("shape", ["rising", "falling", "spike"])
def test_attention_moving_maximum(env, shape):
    """Scores that climb (or fall) steadily along the context, or jump by a large amount at one token:
    the running exponent reference of the softmax has to follow without losing small or large weights."""
    ctx, S, cb = env
    lens = [300, 1000, 3000]
    say(f"attention with {shape} scores, lens={lens}")
    B, Hq, Hkv = len(lens), 4, 1
    g = torch.Generator().manual_seed(900)
    u = torch.randn(128, generator=g, dtype=torch.float64)
    u = u / u.norm()
    # the four heads of the group see the ramp with different slopes and signs
    gains = torch.tensor([1.0, 2.5, -1.0, 0.25], dtype=torch.float64)
    q = (gains[None, :, None] * u[None, None, :] * math.sqrt(128.0)).repeat(B, 1, 1)
    q = (q + 0.05 * torch.randn(q.shape, generator=g, dtype=torch.float64)).to(torch.bfloat16)
    starts, pool = [], 0
    for n in lens:
        starts.append(pool)
        pool += ((n + 63) // 64) * 64
    kc, kr = Context.alloc_cache(Hkv, pool, DEV)
    vc, vr = Context.alloc_cache(Hkv, pool, DEV)
    for t in (kc, kr, vc, vr):
        t.zero_()
    k_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
    v_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
    for b, n in enumerate(lens):
        t = torch.arange(n, dtype=torch.float64) / n
        if shape == "rising":
            c = 40.0 * t
        elif shape == "falling":
            c = 40.0 * (1.0 - t)
        else:
            c = torch.zeros(n, dtype=torch.float64)
            c[(2 * n) // 3] = 30.0
        k = c[:, None] * u[None, :] + torch.randn((n, 128), generator=g, dtype=torch.float64)
        k = k.to(torch.bfloat16)[:, None, :].contiguous()             # [n, 1, 128]
        v = synth.kv_stream(n, Hkv, 901 + b).permute(1, 0, 2).contiguous()
        ctx.encode_kv(k.to(DEV), PQ_KEY, kc, kr, dst_token0=starts[b])
        ctx.encode_kv(v.to(DEV), PQ_VALUE, vc, vr, dst_token0=starts[b])
        k_rec[:, starts[b]:starts[b] + n] = oracle_records(k, S, cb)[0]
        v_rec[:, starts[b]:starts[b] + n] = oracle_records(v, S, cb)[0]
    torch.cuda.synchronize()
    starts = np.array(starts, dtype=np.int64)
    got = gpu_attention(ctx, q, (kc, kr, vc, vr), starts, lens)
    ref = oracle.attention(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb,
                           helpers.softmax_scale())
    assert np.all(np.isfinite(got))
    err = helpers.rel_l2(got, ref)
    per_row = [helpers.rel_l2(got[b, h], ref[b, h]) for b in range(B) for h in range(Hq)]
    say(f"  rel L2 {err:.2e}; worst row {max(per_row):.2e}")
    assert err <= 2e-3


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (16, 2)])
def test_decode_step_equals_append_then_attention(env, Hq, Hkv):
    """pq_decode_step_polar gives, bit for bit, the caches and the output of pq_append_kv_pair followed by
    pq_attn_decode_polar (groups of 4 and of 8 query heads)."""
    ctx, S, cb = env
    lens = [1, 64, 65, 300, 1000]      # context lengths including the token appended in the step
    say(f"decode step vs append + attention, Hq={Hq} Hkv={Hkv} lens={lens}")
    B = len(lens)
    results = []
    for fused in (False, True):
        starts, pool = [], 0
        for n in lens:
            starts.append(pool)
            pool += ((n + 63) // 64) * 64
        kc, kr = Context.alloc_cache(Hkv, pool, DEV)
        vc, vr = Context.alloc_cache(Hkv, pool, DEV)
        for t in (kc, kr, vc, vr):
            t.zero_()
        for b, n in enumerate(lens):
            if n > 1:
                k = synth.kv_stream(n - 1, Hkv, 810 + 2 * b).permute(1, 0, 2).contiguous()
                v = synth.kv_stream(n - 1, Hkv, 811 + 2 * b).permute(1, 0, 2).contiguous()
                ctx.encode_kv(k.to(DEV), PQ_KEY, kc, kr, dst_token0=starts[b])
                ctx.encode_kv(v.to(DEV), PQ_VALUE, vc, vr, dst_token0=starts[b])
        nk = synth.kv_stream(B, Hkv, 830).permute(1, 0, 2).contiguous().to(DEV)
        nv = synth.kv_stream(B, Hkv, 831).permute(1, 0, 2).contiguous().to(DEV)
        q = synth.queries(B, Hq, seed=832).to(DEV)
        seq_start = torch.tensor(starts, dtype=torch.int64, device=DEV)
        ctx_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
        dst = seq_start + ctx_len.to(torch.int64) - 1
        out = torch.empty((B, Hq, 128), dtype=torch.float32, device=DEV)
        ws = torch.empty(Context.attn_workspace_bytes(B, Hq, Hkv, max(lens)), dtype=torch.uint8, device=DEV)
        if fused:
            ctx.decode_step_polar(nk, nv, dst, q, out, kc, kr, vc, vr, seq_start, ctx_len, max(lens),
                                  helpers.softmax_scale(), ws)
        else:
            ctx.append_kv_pair(nk, nv, kc, kr, vc, vr, dst)
            ctx.attn_decode_polar(q, out, kc, kr, vc, vr, seq_start, ctx_len, max(lens), helpers.softmax_scale(), ws)
        torch.cuda.synchronize()
        results.append((kc, kr, vc, vr, out))
    for a, b in zip(*results):
        assert torch.equal(a, b)
    assert torch.isfinite(results[1][4]).all()


def test_decode_step_under_graph_replay(env):
    """The decode step (three launches, no memset nodes, no allocation once the context's tables are on the
    device) captured into a HIP graph: every replay, with eager work and synchronisations in between, gives
    the eager result bit for bit, including after the inputs have changed in place and after the contexts have
    grown (the launch shapes depend on max_ctx only; the work is split on the device from ctx_len)."""
    ctx, S, cb = env
    lens = [70, 300, 1000]
    say(f"decode step under graph replay, lens={lens}")
    B, Hq, Hkv = len(lens), 8, 2
    grow = 70                            # tokens the contexts grow by during the test (crosses a tile boundary)
    caches, starts, pool, _, _ = build_cache(ctx, S, cb, [n + grow for n in lens], Hkv, seed=1700, want_oracle=False)
    kc, kr, vc, vr = caches
    seq_start = torch.from_numpy(starts).to(DEV)
    ctx_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    dst = seq_start + ctx_len.to(torch.int64) - 1
    nk = synth.kv_stream(B, Hkv, 1710).permute(1, 0, 2).contiguous().to(DEV)
    nv = synth.kv_stream(B, Hkv, 1711).permute(1, 0, 2).contiguous().to(DEV)
    q = synth.queries(B, Hq, seed=1712).to(DEV)
    out = torch.empty((B, Hq, 128), dtype=torch.float32, device=DEV)
    max_ctx = max(lens) + grow
    ws = torch.empty(Context.attn_workspace_bytes(B, Hq, Hkv, max_ctx), dtype=torch.uint8, device=DEV)

    def step():
        ctx.decode_step_polar(nk, nv, dst, q, out, kc, kr, vc, vr, seq_start, ctx_len, max_ctx, helpers.softmax_scale(), ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up on a side stream, as graph capture wants it
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for rep in range(6):
        if rep == 2:                    # new query and new token vectors, written in place
            q.copy_(synth.queries(B, Hq, seed=1720).to(DEV))
            nk.copy_(synth.kv_stream(B, Hkv, 1721).permute(1, 0, 2).contiguous().to(DEV))
        if rep >= 3:                    # the contexts grow (by 1, 1 and then to the limit), in place
            step_by = 1 if rep < 5 else grow - 2
            ctx_len.add_(step_by)
            dst.add_(step_by)
        out.fill_(float("nan"))
        step()
        torch.cuda.synchronize()
        eager = out.clone()
        eager_cache = (kc.clone(), kr.clone())
        out.fill_(float("nan"))
        ws.fill_(0xFF)                  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
        assert torch.equal(kc, eager_cache[0]) and torch.equal(kr, eager_cache[1])
    assert torch.isfinite(out).all()


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (2, 2), (16, 2), (6, 2), (12, 2), (5, 1), (16, 1)])
def test_hybrid_attention_prefix_plus_window(env, Hq, Hkv):
    """Quantised prefix + bf16 window against the oracle: every mix of empty / one-tile / ragged prefix and
    empty / partial / several-chunk window."""
    run_hybrid_case(*env, Hq, Hkv)


def run_hybrid_case(ctx, S, cb, Hq, Hkv):
    lens = [0, 1, 0, 100, 1000, 64, 300, 2000]
    wins = [0, 0, 5, 1, 63, 64, 65, 200]
    cap = 200
    say(f"hybrid attention Hq={Hq} Hkv={Hkv} prefix={lens} window={wins}")
    B = len(lens)
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, Hkv, seed=950)
    g = torch.Generator().manual_seed(951)
    win_k = torch.randn((B, Hkv, cap, 128), generator=g).to(torch.bfloat16)
    win_v = torch.randn((B, Hkv, cap, 128), generator=g).to(torch.bfloat16)
    win_k[:, :, :, 7] *= 6.0   # an outlier channel, as in the cached streams
    q = synth.queries(B, Hq, seed=952)
    kc, kr, vc, vr = caches
    out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(Context.attn_hybrid_workspace_bytes(B, Hq, Hkv, max(lens), cap), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    ctx.attn_decode_hybrid(q.to(DEV), out, kc, kr, vc, vr, torch.from_numpy(starts).to(DEV),
                           torch.tensor(lens, dtype=torch.int32, device=DEV), win_k.to(DEV), win_v.to(DEV),
                           torch.tensor(wins, dtype=torch.int32, device=DEV), max(lens), helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.attention_hybrid(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32),
                                  win_k.to(torch.float64).numpy(), win_v.to(torch.float64).numpy(),
                                  np.array(wins, np.int32), S, cb, helpers.softmax_scale())
    assert np.all(np.isfinite(got))
    assert np.all(got[0] == 0.0)                      # neither prefix nor window
    per_seq = [helpers.rel_l2(got[b], ref[b]) for b in range(1, B)]
    err = helpers.rel_l2(got[1:], ref[1:])
    say(f"  rel L2 {err:.2e}; per sequence {['%.1e' % e for e in per_seq]}")
    assert err <= 2e-3 and max(per_seq) <= 4e-3
    # window only (sequence 2): no quantisation in the way, fp32 accuracy
    assert per_seq[1] <= 1e-5
    # the window path with an empty window equals plain attention on the prefix, bit for bit
    out2 = torch.empty_like(out)
    ctx.attn_decode_hybrid(q.to(DEV), out2, kc, kr, vc, vr, torch.from_numpy(starts).to(DEV),
                           torch.tensor(lens, dtype=torch.int32, device=DEV), win_k.to(DEV), win_v.to(DEV),
                           torch.zeros(B, dtype=torch.int32, device=DEV), max(lens), helpers.softmax_scale(), ws)
    plain = gpu_attention(ctx, q, caches, starts, lens)
    torch.cuda.synchronize()
    assert helpers.rel_l2(out2.cpu().numpy()[1:], plain[1:]) <= 1e-6


@pytest.mark.parametrize("which", ["hadamard", "identity"])
def test_other_preconditioners_encode_and_attend(which):
    """A randomised Hadamard S (one exact bf16 term in the encode kernel) and S = I (no preconditioning):
    the library's S is handed to the oracle as data; encode, DeQuant and attention against it."""
    cb = oracle.default_codebooks()
    if which == "hadamard":
        ctx = Context(seed=5, hadamard=True)
    else:
        ctx = Context(S=np.eye(128))
    S = ctx.preconditioner()
    assert np.max(np.abs(S @ S.T - np.eye(128))) <= 1e-12
    for kind in (PQ_KEY, PQ_VALUE):
        if which == "hadamard":
            for dtype in (torch.bfloat16, torch.float32):
                x = synth.kv_stream(700, 3, seed=970 + kind).permute(1, 0, 2).contiguous().to(dtype)
                check_encode(ctx, S, cb, x, kind, f"{which} S")
        else:
            # without a rotation, 8-bit mantissas would put 0.25 % of the level-1 pairs exactly on the pi/4
            # boundaries (|y_2j| == |y_2j+1|), where either neighbour is a correct code: full fp32 data here
            x = synth.gaussian_vectors(700 * 3, seed=972 + kind).reshape(700, 3, 128)
            check_encode(ctx, S, cb, x, kind, f"{which} S")
    lens = [1, 200, 1500]
    if which == "hadamard":
        caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, 2, seed=980)
    else:
        # plain N(0,1) keys and values: without the rotation the outlier channels of the usual streams
        # make the scores several times larger and the softmax correspondingly more sensitive, which is
        # the regime the preconditioner exists to avoid, not the one the 2e-3 bound is stated for
        Hkv, starts, pool = 2, [], 0
        for n in lens:
            starts.append(pool)
            pool += ((n + 63) // 64) * 64
        kc, kr = Context.alloc_cache(Hkv, pool, DEV)
        vc, vr = Context.alloc_cache(Hkv, pool, DEV)
        for t in (kc, kr, vc, vr):
            t.zero_()
        k_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
        v_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
        for b, n in enumerate(lens):
            k = synth.gaussian_vectors(n * Hkv, seed=982 + 2 * b).reshape(n, Hkv, 128)
            v = synth.gaussian_vectors(n * Hkv, seed=983 + 2 * b).reshape(n, Hkv, 128)
            ctx.encode_kv(k.to(DEV), PQ_KEY, kc, kr, dst_token0=starts[b])
            ctx.encode_kv(v.to(DEV), PQ_VALUE, vc, vr, dst_token0=starts[b])
            k_rec[:, starts[b]:starts[b] + n] = oracle_records(k, S, cb)[0]
            v_rec[:, starts[b]:starts[b] + n] = oracle_records(v, S, cb)[0]
        torch.cuda.synchronize()
        caches, starts = (kc, kr, vc, vr), np.array(starts, dtype=np.int64)
    q = synth.queries(len(lens), 8, seed=981)
    got = gpu_attention(ctx, q, caches, starts, lens)
    ref = oracle.attention(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb,
                           helpers.softmax_scale())
    err = helpers.rel_l2(got, ref)
    say(f"  {which} S: attention rel L2 {err:.2e}")
    assert err <= 2e-3


@pytest.fixture(scope="module", params=["generated", "handed_in"])
def hadamard_env(request):
    """A context whose S is a sign diagonal times the Sylvester Hadamard matrix, made by the library or handed in
    as a plain matrix: either way the single-vector products with S run as fast Walsh-Hadamard transforms.  The
    oracle gets the library's S as data and multiplies by it as by any other matrix."""
    ctx = Context(seed=5, hadamard=True)
    if request.param == "handed_in":
        ctx = Context(S=ctx.preconditioner())
    assert ctx.preconditioner_structure() == 2
    return ctx, ctx.preconditioner(), oracle.default_codebooks()


def test_hadamard_append(hadamard_env):
    """Appended keys and values (transform of D x, the factor 1/sqrt(128) taken into the radius) against the oracle."""
    run_append_case(*hadamard_env)


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (6, 2)])
def test_hadamard_hybrid_attention(hadamard_env, Hq, Hkv):
    """Query rotation and un-rotation of the output by the transform, in the launch that also scores the window."""
    run_hybrid_case(*hadamard_env, Hq, Hkv)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_hadamard_decode_step(hadamard_env, dtype):
    """One decode step (append + query rotation + attention + un-rotation) against the oracle: the prefix is the
    oracle's own records, the new token is encoded by both sides (records compared under the tie rule) and the
    output is compared with the oracle's attention over its records of all tokens."""
    ctx, S, cb = hadamard_env
    Hq, Hkv = 8, 2
    lens = [1, 64, 65, 300, 1000]      # context lengths including the token appended in the step
    say(f"Hadamard S: decode step, {dtype}, lens={lens}")
    B = len(lens)
    starts, pool = [], 0
    for n in lens:
        starts.append(pool)
        pool += ((n + 63) // 64) * 64
    kc, kr = Context.alloc_cache(Hkv, pool, DEV)
    vc, vr = Context.alloc_cache(Hkv, pool, DEV)
    for t in (kc, kr, vc, vr):
        t.zero_()
    k_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
    v_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
    nk = synth.kv_stream(B, Hkv, 1830).permute(1, 0, 2).contiguous().to(dtype)     # [B, Hkv, 128]
    nv = synth.kv_stream(B, Hkv, 1831).permute(1, 0, 2).contiguous().to(dtype)
    psi_new, y_new = {}, {}
    for b, n in enumerate(lens):
        for kind, codes, radii, rec, new, seed in ((PQ_KEY, kc, kr, k_rec, nk, 1810), (PQ_VALUE, vc, vr, v_rec, nv, 1811)):
            if n > 1:
                old = synth.kv_stream(n - 1, Hkv, seed + 2 * b).permute(1, 0, 2).contiguous()
                rec_old = oracle_records(old, S, cb)[0]
                rec[:, starts[b] : starts[b] + n - 1] = rec_old
                helpers.upload_records(kind, rec_old, codes, radii, starts[b])
            rec_new, psi, y = oracle_records(new[b : b + 1], S, cb)
            rec[:, starts[b] + n - 1] = rec_new[:, 0]
            psi_new[(kind, b)], y_new[(kind, b)] = psi[:, 0], y[:, 0]
    q = synth.queries(B, Hq, seed=1832)
    seq_start = torch.tensor(starts, dtype=torch.int64, device=DEV)
    ctx_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    dst = seq_start + ctx_len.to(torch.int64) - 1
    out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(Context.attn_workspace_bytes(B, Hq, Hkv, max(lens)), dtype=torch.uint8, device=DEV)
    ctx.decode_step_polar(nk.to(DEV), nv.to(DEV), dst, q.to(DEV), out, kc, kr, vc, vr, seq_start, ctx_len, max(lens),
                          helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    # the appended records
    n_bad = 0
    for kind, codes, radii, rec in ((PQ_KEY, kc, kr, k_rec), (PQ_VALUE, vc, vr, v_rec)):
        for b, n in enumerate(lens):
            slot = starts[b] + n - 1
            got = canonical_both_ways(ctx, kind, codes, radii, slot - slot % 64, 64)[:, slot % 64]
            st, rg, ro = helpers.check_codes(got.reshape(-1, 62), rec[:, slot].reshape(-1, 62),
                                             psi_new[(kind, b)].reshape(-1, 120), enforce_rate=False)
            helpers.check_radii(rg, ro, y_new[(kind, b)].reshape(-1, 128), enforce_rate=False)
            n_bad += st["code_mismatches"]
    assert n_bad <= 1       # 2400 angles: a single proven tie at most
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.attention(q.to(torch.float64).numpy(), k_rec, v_rec, np.array(starts, np.int64), np.array(lens, np.int32),
                           S, cb, helpers.softmax_scale())
    err = helpers.rel_l2(got, ref)
    per_seq = [helpers.rel_l2(got[b], ref[b]) for b in range(B)]
    say(f"  rel L2 {err:.2e}; per sequence {['%.1e' % e for e in per_seq]}; appended-code ties {n_bad}")
    assert np.all(np.isfinite(got))
    assert err <= 2e-3 and max(per_seq) <= 4e-3


def lloyd_1d(samples, init, iters=8):
    """Plain 1-D Lloyd iterations (nearest centroid by linear distance, centroid = mean of its cell)."""
    c = np.array(init, dtype=np.float64)
    for _ in range(iters):
        edges = 0.5 * (c[:-1] + c[1:])
        idx = np.searchsorted(edges, samples)
        for k in range(c.size):
            sel = samples[idx == k]
            if sel.size:
                c[k] = sel.mean()
    return c


@pytest.mark.parametrize("which", ["jittered", "fitted_no_rotation", "jittered_hadamard"])
def test_general_codebooks_encode_and_attend(which):
    """Codebooks set by the caller (pq_set_codebooks): the analytic ones moved at random, and codebooks fitted
    by Lloyd iterations to the angles of un-rotated data with outlier channels (S = I, the paper's variant
    without preconditioning).  Encode (bulk and append), DeQuant and attention against the oracle, which
    takes the same centroids as data."""
    cb = oracle.default_codebooks().copy()
    if which in ("jittered", "jittered_hadamard"):
        # with a Hadamard S the encode kernel's one-term product and the transform paths meet the level-1 cell table
        ctx = Context(seed=3, hadamard=(which == "jittered_hadamard"))
        rng = np.random.default_rng(11)
        cb[:16] += rng.uniform(-0.08, 0.08, 16)
        cb[16:] += rng.uniform(-0.04, 0.04, 12)
        make = lambda n, H, seed: synth.kv_stream(n, H, seed).permute(1, 0, 2).contiguous()
    else:
        ctx = Context(S=np.eye(128))
        # fp32 data with three strong channels: level-1 angles of the pairs that hold them crowd the axes
        def make(n, H, seed):
            x = synth.gaussian_vectors(n * H, seed=seed).reshape(n, H, 128).clone()
            x[:, :, [5, 40, 99]] *= 6.0
            return x
        sample = make(4096, 1, 990).reshape(-1, 128).double().numpy()
        _, psi, _ = oracle.encode(sample, np.eye(128), cb, want_psi=True, want_y=True)
        psi = psi.reshape(-1, 120)
        cb[:16] = lloyd_1d(psi[:, :64].ravel(), cb[:16])
        cb[16:20] = lloyd_1d(psi[:, 64:96].ravel(), cb[16:20])
        cb[20:24] = lloyd_1d(psi[:, 96:112].ravel(), cb[20:24])
        cb[24:28] = lloyd_1d(psi[:, 112:120].ravel(), cb[24:28])
    ctx.set_codebooks(cb)
    S = ctx.preconditioner()
    say(f"general codebooks ({which}): level-1 centroids {np.round(cb[:16], 3).tolist()}")
    for kind in (PQ_KEY, PQ_VALUE):
        x = make(700, 3, 991 + kind)
        codes, radii, rec_gpu, rec_or = check_encode(ctx, S, cb, x, kind, f"{which} codebooks")
        # DeQuant on identical codes: the oracle's records laid out as tiles
        codes_or, radii_or = Context.alloc_cache(3, 704, DEV)
        helpers.upload_records(kind, rec_or, codes_or, radii_or, 0)
        out = torch.empty((700, 3, 128), dtype=torch.float32, device=DEV)
        ctx.decode_kv(kind, codes_or, radii_or, 0, 700, out, rotated=False)
        torch.cuda.synchronize()
        ref = oracle.decode(rec_or.reshape(-1, 62), S, cb).reshape(3, 700, 128)
        assert helpers.rel_l2(out.cpu().numpy().transpose(1, 0, 2), ref) <= 1e-5
        # append of one more token goes through the same codebooks
        new = make(2, 3, 995 + kind)[:1].contiguous()            # [1, 3, 128]
        ctx.append_kv(new.to(DEV), kind, codes, radii, torch.tensor([700], dtype=torch.int64, device=DEV))
        torch.cuda.synchronize()
        rec = canonical_both_ways(ctx, kind, codes, radii, 640, 64)[:, 700 - 640]
        rec_o, psi_o, y_o = oracle_records(new, S, cb)
        st, rg, ro = helpers.check_codes(rec.reshape(-1, 62), rec_o.reshape(-1, 62), psi_o.reshape(-1, 120), cb=cb)
        helpers.check_radii(rg, ro, y_o.reshape(-1, 128))
    # attention
    lens, Hkv = [70, 900], 2
    starts, pool = [], 0
    for n in lens:
        starts.append(pool)
        pool += ((n + 63) // 64) * 64
    kc, kr = Context.alloc_cache(Hkv, pool, DEV)
    vc, vr = Context.alloc_cache(Hkv, pool, DEV)
    for t in (kc, kr, vc, vr):
        t.zero_()
    k_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
    v_rec = np.zeros((Hkv, pool, 62), dtype=np.uint8)
    for b, n in enumerate(lens):
        k, v = make(n, Hkv, 996 + 2 * b), make(n, Hkv, 997 + 2 * b)
        ctx.encode_kv(k.to(DEV), PQ_KEY, kc, kr, dst_token0=starts[b])
        ctx.encode_kv(v.to(DEV), PQ_VALUE, vc, vr, dst_token0=starts[b])
        k_rec[:, starts[b]:starts[b] + n] = oracle_records(k, S, cb)[0]
        v_rec[:, starts[b]:starts[b] + n] = oracle_records(v, S, cb)[0]
    torch.cuda.synchronize()
    starts = np.array(starts, dtype=np.int64)
    q = synth.queries(len(lens), 8, seed=998)
    got = gpu_attention(ctx, q, (kc, kr, vc, vr), starts, lens)
    ref = oracle.attention(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb,
                           helpers.softmax_scale())
    err = helpers.rel_l2(got, ref)
    say(f"  {which} codebooks: attention rel L2 {err:.2e}")
    assert err <= 2e-3


@pytest.mark.parametrize("which", ["rotated", "no_rotation", "hadamard"])
def test_online_codebook_fit(which):
    """pq_fit_codebooks against the oracle's k-means on the exact angles: the GPU counts the angles into
    fine histograms and clusters the bins, so the centroids agree to a fraction of a bin width; the fitted
    codebooks then drive encode with bit-exact codes."""
    base = oracle.default_codebooks()
    if which == "rotated":
        ctx = Context(seed=2)
        x = synth.kv_stream(5000, 2, seed=60).permute(1, 0, 2).contiguous()          # bf16, outlier channels
        x[4990:] *= 0.0                                                               # some all-zero vectors
    elif which == "hadamard":
        # the kernel multiplies by sqrt(128) S (entries +-1, one exact bf16 term): the angles do not see the factor
        ctx = Context(seed=2, hadamard=True)
        x = synth.kv_stream(4000, 2, seed=62).permute(1, 0, 2).contiguous()
    else:
        ctx = Context(S=np.eye(128))
        x = synth.gaussian_vectors(2 * 3001, seed=61).reshape(3001, 2, 128).clone()   # fp32, ragged tile tail
        x[:, :, [5, 40, 99]] *= 6.0
    S = ctx.preconditioner()
    iters = 6
    say(f"online codebook fit ({which}): {x.shape[0]} tokens x {x.shape[1]} heads, {iters} rounds")
    got = ctx.fit_codebooks(x.to(DEV), iters)
    ref = oracle.fit_codebooks(x.reshape(-1, 128).double().numpy(), S, base, iters)
    d1, du = np.max(np.abs(got[:16] - ref[:16])), np.max(np.abs(got[16:] - ref[16:]))
    # the library counts angles in bins uniform in the pseudo-angle v / (u + v): 4.9e-4 to 9.8e-4 rad wide
    say(f"  max centroid difference: level 1 {d1:.2e} rad, levels 2-4 {du:.2e} rad (bins 4.9e-4 .. 9.8e-4 rad)")
    assert d1 <= 3e-4 and du <= 3e-4
    if which == "no_rotation":
        assert np.max(np.abs(got[:16] - base[:16])) > 0.005      # the data moved the level-1 codebook
    # zero rounds give the start back; an explicit start is honoured
    assert np.max(np.abs(ctx.fit_codebooks(x.to(DEV), 0) - base)) <= 1e-12   # the library's own analytic codebooks
    start = base.copy(); start[16:20] += 0.01
    assert np.array_equal(ctx.fit_codebooks(x.to(DEV), 0, cb_init=start), start)
    # a context with fitted codebooks (the oracle's) encodes bit-exactly against the oracle using them
    ctx2 = Context(S=S)
    ctx2.set_codebooks(ref)
    xs = x[:700].contiguous()
    check_encode(ctx2, S, ref, xs, PQ_KEY, f"fitted ({which})")


@pytest.mark.parametrize("M,Hq,Hkv", [(2, 8, 2), (4, 4, 1), (3, 2, 2), (16, 1, 1), (1, 16, 2), (2, 16, 2), (2, 6, 2), (3, 5, 1),
                                      (2, 7, 1), (1, 16, 1)])
def test_multi_query_attention(env, M, Hq, Hkv):
    """M query tokens per sequence (and 8 query heads per kv head): row (b, m) equals single-query attention
    over the first ctx_len - (M-1-m) cached tokens -- the oracle is called once per m with that length."""
    ctx, S, cb = env
    lens = [M, 64, 65 + M, 130, 1000, 64 * 5 + 1]      # tile boundaries inside the M newest tokens
    say(f"multi-query attention M={M} Hq={Hq} Hkv={Hkv} lens={lens}")
    B = len(lens)
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, Hkv, seed=1100 + M)
    kc, kr, vc, vr = caches
    q = synth.queries(B * M, Hq, seed=1101).reshape(B, M, Hq, 128).contiguous()
    out = torch.full((B, M, Hq, 128), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(Context.attn_mq_workspace_bytes(B, M, Hq, Hkv, max(lens)), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    ctx.attn_decode_polar_mq(q.to(DEV), out, kc, kr, vc, vr, torch.from_numpy(starts).to(DEV),
                             torch.tensor(lens, dtype=torch.int32, device=DEV), max(lens), helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    errs = []
    for m in range(M):
        lens_m = np.array([max(n - (M - 1 - m), 0) for n in lens], dtype=np.int32)
        ref = oracle.attention(q[:, m].to(torch.float64).numpy(), k_rec, v_rec, starts, lens_m, S, cb,
                               helpers.softmax_scale())
        errs.append(helpers.rel_l2(got[:, m], ref))
        for b in range(B):
            if lens_m[b] == 0:
                assert np.all(got[b, m] == 0.0)
            else:
                assert helpers.rel_l2(got[b, m], ref[b]) <= 2e-3, (b, m)
    say(f"  rel L2 per query token {['%.1e' % e for e in errs]}")
    assert max(errs) <= 2e-3
    if M == 1:   # the multi-query entry point with one token is the plain one
        plain = gpu_attention(ctx, q[:, 0], caches, starts, lens)
        assert np.array_equal(plain, out[:, 0].cpu().numpy())


def test_attention_rejects_bad_sequences_gracefully(env):
    ctx, S, cb = env
    say("attention with an unaligned / out-of-pool sequence")
    lens = [100, 100]
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, 1, seed=700, want_oracle=False)
    q = synth.queries(2, 4, seed=700)
    bad_starts = starts.copy()
    bad_starts[1] = pool  # outside the pool: treated as empty, never read
    got = gpu_attention(ctx, q, caches, bad_starts, lens)
    assert np.all(np.isfinite(got)) and np.all(got[1] == 0.0)


def test_attention_rejects_more_than_sixteen_heads_per_kv_head(env):
    """17 query heads per kv head do not fit the 16 (query token, head) pairs of a pass: refused on the host,
    nothing launched, the output untouched."""
    ctx, S, cb = env
    say("attention with Hq/Hkv = 17: refused")
    lens = [100]
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, lens, 1, seed=701, want_oracle=False)
    q = synth.queries(1, 17, seed=701)
    with pytest.raises(Exception) as e:
        gpu_attention(ctx, q, caches, starts, lens)
    assert "-2" in str(e.value) or "UNSUPPORTED" in str(e.value).upper()
