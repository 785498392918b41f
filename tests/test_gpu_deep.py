"""GPU parity of the full-depth recursion (L = 7, one radius per vector) against the fp64 oracle.

Every input is seeded and synthetic.  Each test prints what it is about to run before touching the GPU.
"""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2502_02617_amd import Context, PQ_KEY, PQ_VALUE, PolarQuantError, synth
from tests import helpers, layout_ref

pytestmark = pytest.mark.gpu
DEV = "cuda"
BITS = [(2, 2, 2), (3, 1, 1), (1, 3, 2)]


def say(msg):
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


def make(bits, **kw):
    ctx = Context(seed=0, **kw)
    ctx.set_recursion_depth(7, bits)
    S = ctx.preconditioner() if kw else oracle.preconditioner(0)
    return ctx, S, oracle.default_codebooks(), oracle.upper_codebooks(bits)


def export_both_ways(ctx, kind, codes, top, token0, n_tokens):
    """50-byte records via the library's export kernel and via the independent numpy reading of the layout."""
    H = codes.shape[0]
    rec = torch.empty((H, n_tokens, 50), dtype=torch.uint8, device=DEV)
    ctx.export_canonical(kind, codes, top, token0, n_tokens, rec)
    torch.cuda.synchronize()
    rec_lib = rec.cpu().numpy()
    c = codes.cpu().numpy()
    t = top.cpu().numpy().view(np.uint16)
    assert token0 % 64 == 0
    t0 = token0 // 64
    rec_np = np.stack([layout_ref.tiles_to_canonical_deep(kind, c[h, t0:], t[h, t0:], n_tokens) for h in range(H)])
    assert np.array_equal(rec_lib, rec_np), "export kernel and layout specification disagree"
    return rec_lib


def oracle_records(x_cpu, S, cb, bits, cbt):
    """x_cpu [T, H, 128] -> records [H, T, 50], psi [H, T, 127], y [H, T, 128]."""
    T, H, _ = x_cpu.shape
    xs = x_cpu.permute(1, 0, 2).contiguous().to(torch.float64).numpy().reshape(H * T, 128)
    rec, psi, y = oracle.encode_deep(xs, S, cb, bits, cbt, want_psi=True, want_y=True)
    return rec.reshape(H, T, 50), psi.reshape(H, T, 127), y.reshape(H, T, 128)


def check_records(rec_gpu, rec_or, psi, y, bits):
    st, rg, ro = helpers.check_codes_deep(rec_gpu.reshape(-1, 50), rec_or.reshape(-1, 50), psi.reshape(-1, 127), bits)
    st.update(helpers.check_radii_deep(rg, ro, y.reshape(-1, 128)))
    return st


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("kind", [PQ_KEY, PQ_VALUE])
def test_deep_encode_and_dequant(bits, kind):
    ctx, S, cb, cbt = make(bits)
    assert ctx.recursion_depth() == 7 and ctx.radii_halves_per_tile() == 128 and ctx.record_bytes() == 50
    for dtype, T, H in ((torch.bfloat16, 1000 + 37, 2), (torch.float32, 300, 1)):
        say(f"deep encode bits={bits} kind={kind} dtype={dtype} T={T} H={H}")
        if dtype == torch.bfloat16:
            x = synth.kv_stream(T, H, seed=41 + kind).permute(1, 0, 2).contiguous()     # [T, H, 128] bf16, outlier channels
        else:
            x = synth.gaussian_vectors(T * H, seed=43).reshape(T, H, 128)
        pool = ((T + 63) // 64) * 64
        codes, top = ctx.alloc_cache_for(H, pool, DEV)
        codes.fill_(0xA5)
        top.fill_(0x5A5A)
        ctx.encode_kv(x.to(DEV), kind, codes, top)
        torch.cuda.synchronize()
        rec_gpu = export_both_ways(ctx, kind, codes, top, 0, T)
        rec_or, psi, y = oracle_records(x, S, cb, bits, cbt)
        say(f"  {check_records(rec_gpu, rec_or, psi, y, bits)}")
        # slots after the input keep their old bytes
        if T % 64:
            tail = export_both_ways(ctx, kind, codes, top, (T // 64) * 64, 64)[:, T % 64:]
            assert np.all(tail[:, :, 46:] == 0x5A)
        # DeQuant on identical codes (the oracle's records laid out as tiles) and end to end
        codes_or, top_or = ctx.alloc_cache_for(H, pool, DEV)
        helpers.upload_records_deep(kind, rec_or, codes_or, top_or, 0)
        out = torch.empty((T, H, 128), dtype=torch.float32, device=DEV)
        out_or = torch.empty_like(out)
        for rotated in (True, False):
            ctx.decode_kv(kind, codes, top, 0, T, out, rotated=rotated)
            ctx.decode_kv(kind, codes_or, top_or, 0, T, out_or, rotated=rotated)
            torch.cuda.synchronize()
            got, got_same = out.cpu().numpy(), out_or.cpu().numpy()
            for h in range(H):
                ref = oracle.decode_deep(rec_or[h], S, cb, bits, cbt, rotated=rotated)
                e_same, e_or = helpers.rel_l2(got_same[:, h], ref), helpers.rel_l2(got[:, h], ref)
                assert e_same <= 1e-5 and e_or <= 1e-3, (rotated, h, e_same, e_or)


def test_deep_encode_hadamard_preconditioner():
    bits = (2, 2, 2)
    ctx, S, cb, cbt = make(bits, hadamard=True)
    T, H = 200, 2
    say(f"deep encode with a randomised Hadamard S: T={T} H={H}")
    x = synth.kv_stream(T, H, seed=47).permute(1, 0, 2).contiguous()
    codes, top = ctx.alloc_cache_for(H, 256, DEV)
    codes.zero_()
    top.zero_()
    ctx.encode_kv(x.to(DEV), PQ_KEY, codes, top)
    torch.cuda.synchronize()
    rec_gpu = export_both_ways(ctx, PQ_KEY, codes, top, 0, T)
    rec_or, psi, y = oracle_records(x, S, cb, bits, cbt)
    say(f"  {check_records(rec_gpu, rec_or, psi, y, bits)}")


@pytest.mark.parametrize("bits,upper", [((2, 2, 2), False), ((2, 2, 2), True), ((3, 1, 2), True)])
def test_deep_with_caller_set_codebooks(bits, upper):
    """Full depth together with codebooks replaced for levels 1-4 (jittered centroids) and, with
    upper, for levels 5-7 as well: encode, append and DeQuant follow them."""
    rng = np.random.default_rng(77)
    cb = oracle.default_codebooks()
    cb[:16] += rng.uniform(-0.05, 0.05, 16)
    cb[16:] += rng.uniform(-0.03, 0.03, 12)
    ctx = Context(seed=0)
    ctx.set_codebooks(cb)
    ctx.set_recursion_depth(7, bits)
    S, cbt = oracle.preconditioner(0), oracle.upper_codebooks(bits)
    if upper:
        for l in range(3):
            K = 1 << bits[l]
            cbt[l, :K] += rng.uniform(-0.01, 0.01, K)
        ctx.set_upper_codebooks(cbt)
        for l in range(3):
            got_bits, cen, bnd = ctx.upper_codebook(5 + l)
            K = 1 << bits[l]
            assert got_bits == bits[l] and np.array_equal(cen[:K], cbt[l, :K])
            assert np.allclose(bnd[1:K], 0.5 * (cbt[l, :K - 1] + cbt[l, 1:K]), rtol=0, atol=1e-15)
    T, H = 500, 2
    say(f"deep + caller-set codebooks: T={T} H={H}")
    caches, records = {}, {}
    for kind in (PQ_KEY, PQ_VALUE):
        x = synth.kv_stream(T, H, seed=81 + kind).permute(1, 0, 2).contiguous()
        codes, top = ctx.alloc_cache_for(H, 512, DEV)
        codes.zero_()
        top.zero_()
        ctx.encode_kv(x[:490].to(DEV), kind, codes, top)
        ctx.append_kv(x[490:].to(DEV).reshape(10, H, 128)[:1].contiguous(), kind, codes, top,
                      torch.tensor([490], dtype=torch.int64, device=DEV))
        torch.cuda.synchronize()
        rec_gpu = export_both_ways(ctx, kind, codes, top, 0, 491)
        rec_or, psi, y = oracle_records(x[:491], S, cb, bits, cbt)
        # boundary distances are those of the jittered codebooks: compare codes directly, allow the tie rate
        Jg, rg = layout_ref.unpack_canonical_deep(rec_gpu.reshape(-1, 50), bits)
        Jo, ro = oracle.unpack_deep(rec_or.reshape(-1, 50), bits)
        bad = Jg != Jo
        say(f"  kind {kind}: {int(bad.sum())} code mismatches of {Jo.size}, {int((rg != ro).sum())} radius mismatches")
        if bad.any():
            tables = [cb[0:16], cb[16:20], cb[20:24], cb[24:28], cbt[0, :1 << bits[0]], cbt[1, :1 << bits[1]],
                      cbt[2, :1 << bits[2]]]
            level = np.concatenate([np.full(64, 0), np.full(32, 1), np.full(16, 2), np.full(8, 3), np.full(4, 4), np.full(2, 5), [6]])
            psi2 = psi.reshape(-1, 127)
            for n_, a_ in zip(*np.nonzero(bad)):
                t = tables[level[a_]]
                mids = 0.5 * (t[:-1] + t[1:])
                assert np.min(np.abs(mids - psi2[n_, a_])) <= helpers.ANGLE_TOL
        assert bad.mean() <= helpers.CODE_MISMATCH_RATE
        helpers.check_radii_deep(rg, ro, y.reshape(-1, 128))
        # DeQuant and (below) attention on identical codes: the oracle's records laid out as tiles
        codes_or, top_or = ctx.alloc_cache_for(H, 512, DEV)
        helpers.upload_records_deep(kind, rec_or, codes_or, top_or, 0)
        out = torch.empty((491, H, 128), dtype=torch.float32, device=DEV)
        ctx.decode_kv(kind, codes_or, top_or, 0, 491, out)
        torch.cuda.synchronize()
        for h in range(H):
            assert helpers.rel_l2(out.cpu().numpy()[:, h], oracle.decode_deep(rec_or[h], S, cb, bits, cbt)) <= 1e-5
        caches[kind], records[kind] = (codes_or, top_or), rec_or
    # attention on the two caches against the oracle on the same records
    n, Hq = 491, 4 * H
    q = synth.queries(1, Hq, seed=83)
    out = torch.empty((1, Hq, 128), dtype=torch.float32, device=DEV)
    ws = torch.empty(Context.attn_workspace_bytes(1, Hq, H, n), dtype=torch.uint8, device=DEV)
    ctx.attn_decode_polar(q.to(DEV), out, caches[PQ_KEY][0], caches[PQ_KEY][1], caches[PQ_VALUE][0], caches[PQ_VALUE][1],
                          torch.zeros(1, dtype=torch.int64, device=DEV), torch.tensor([n], dtype=torch.int32, device=DEV),
                          n, helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    ref = oracle.attention_deep(q.to(torch.float64).numpy(), records[PQ_KEY], records[PQ_VALUE], np.zeros(1, np.int64),
                                np.array([n], np.int32), S, cb, bits, cbt, helpers.softmax_scale())
    err = helpers.rel_l2(out.cpu().numpy(), ref)
    say(f"  attention rel L2 {err:.2e}")
    assert err <= 2e-3


@pytest.mark.parametrize("bits", [(2, 2, 2), (3, 1, 2)])
def test_deep_online_codebook_fit(bits):
    """pq_fit_codebooks_deep against the oracle's k-means on the exact angles, all seven levels; the fitted
    codebooks then drive a fresh context whose codes match the oracle's with the same codebooks."""
    ctx = Context(seed=3)
    ctx.set_recursion_depth(7, bits)
    S = ctx.preconditioner()
    x = synth.kv_stream(6000, 2, seed=70).permute(1, 0, 2).contiguous()          # bf16, outlier channels
    x[5990:] *= 0.0                                                               # some all-zero vectors
    iters = 6
    say(f"deep online codebook fit bits={bits}: {x.shape[0]} tokens x {x.shape[1]} heads, {iters} rounds")
    base, base_t = oracle.default_codebooks(), oracle.upper_codebooks(bits)
    got, got_t = ctx.fit_codebooks_deep(x.to(DEV), iters)
    xs = x.reshape(-1, 128).double().numpy()
    ref = oracle.fit_codebooks(xs, S, base, iters)
    ref_t = oracle.fit_upper_codebooks(xs, S, bits, base_t, iters)
    d_low = np.max(np.abs(got - ref))
    d_up = max(np.max(np.abs(got_t[l, :1 << bits[l]] - ref_t[l, :1 << bits[l]])) for l in range(3))
    say(f"  max centroid difference: levels 1-4 {d_low:.2e} rad, levels 5-7 {d_up:.2e} rad (bins 4.9e-4 .. 9.8e-4 rad)")
    assert d_low <= 3e-4 and d_up <= 3e-4
    # zero rounds give the start back; an explicit start is honoured
    z, z_t = ctx.fit_codebooks_deep(x.to(DEV), 0)
    assert np.max(np.abs(z - base)) <= 1e-12
    assert all(np.max(np.abs(z_t[l, :1 << bits[l]] - base_t[l, :1 << bits[l]])) <= 1e-12 for l in range(3))
    start_t = base_t.copy()
    start_t[0, :1 << bits[0]] += 0.004
    assert np.array_equal(ctx.fit_codebooks_deep(x.to(DEV), 0, cbt_init=start_t)[1], start_t)
    with pytest.raises(PolarQuantError):
        Context(seed=3).fit_codebooks_deep(x.to(DEV), 1)     # not a depth-7 context
    # a fresh context with fitted codebooks (the oracle's) encodes like the oracle with them
    ctx2 = Context(S=S)
    ctx2.set_codebooks(ref)
    ctx2.set_recursion_depth(7, bits)
    ctx2.set_upper_codebooks(ref_t)
    T, H = 700, 2
    xe = x[:T].contiguous()
    codes, top = ctx2.alloc_cache_for(H, 704, DEV)
    codes.zero_()
    top.zero_()
    ctx2.encode_kv(xe.to(DEV), PQ_KEY, codes, top)
    torch.cuda.synchronize()
    rec_gpu = export_both_ways(ctx2, PQ_KEY, codes, top, 0, T)
    rec_or, psi, y = oracle_records(xe, S, ref, bits, ref_t)
    Jg, rg = layout_ref.unpack_canonical_deep(rec_gpu.reshape(-1, 50), bits)
    Jo, ro = oracle.unpack_deep(rec_or.reshape(-1, 50), bits)
    bad = Jg != Jo
    say(f"  encode with the fitted codebooks: {int(bad.sum())} code mismatches of {Jo.size}")
    assert bad.mean() <= helpers.CODE_MISMATCH_RATE
    helpers.check_radii_deep(rg, ro, y.reshape(-1, 128))


@pytest.mark.parametrize("hadamard", [False, True])
def test_deep_offsets_and_append(hadamard):
    """hadamard: the appended vector is rotated by a fast Walsh-Hadamard transform, the factor 1/sqrt(128) goes
    into the vector's one radius."""
    bits = (2, 2, 2)
    ctx, S, cb, cbt = make(bits, hadamard=True) if hadamard else make(bits)
    H, pool = 2, 256
    say(f"deep: encode into the middle of a tile, then append single tokens (Hadamard S: {hadamard})")
    x = synth.kv_stream(90, H, seed=51).permute(1, 0, 2).contiguous()        # [90, H, 128]
    codes, top = ctx.alloc_cache_for(H, pool, DEV)
    codes.zero_()
    top.zero_()
    for kind in (PQ_KEY, PQ_VALUE):
        codes.zero_()
        top.zero_()
        ctx.encode_kv(x[:70].to(DEV), kind, codes, top, dst_token0=20)       # slots 20..89: two partial tiles
        for t in range(70, 90):                                              # slots 90..109 one at a time
            ctx.append_kv(x[t:t + 1].to(DEV), kind, codes, top, torch.tensor([20 + t], dtype=torch.int64, device=DEV))
        torch.cuda.synchronize()
        rec_gpu = export_both_ways(ctx, kind, codes, top, 0, 128)
        rec_or, psi, y = oracle_records(x, S, cb, bits, cbt)
        say(f"  kind {kind}: {check_records(rec_gpu[:, 20:110], rec_or, psi, y, bits)}")
        assert np.all(rec_gpu[:, :20] == 0) and np.all(rec_gpu[:, 110:] == 0)


def build_cache(ctx, S, cb, bits, cbt, lens, Hkv, seed):
    starts, pool = [], 0
    for n in lens:
        starts.append(pool)
        pool += ((max(n, 1) + 63) // 64) * 64
    kc, kt = ctx.alloc_cache_for(Hkv, pool, DEV)
    vc, vt = ctx.alloc_cache_for(Hkv, pool, DEV)
    for t in (kc, vc):
        t.fill_(0xFF)
    for t in (kt, vt):
        t.fill_(0x7E00)    # stale slots: binary16 NaN radius, arbitrary codes
    k_rec = np.zeros((Hkv, pool, 50), dtype=np.uint8)
    v_rec = np.zeros((Hkv, pool, 50), dtype=np.uint8)
    for b, n in enumerate(lens):
        if n == 0:
            continue
        k = synth.kv_stream(n, Hkv, seed + 2 * b).permute(1, 0, 2).contiguous()
        v = synth.kv_stream(n, Hkv, seed + 2 * b + 1).permute(1, 0, 2).contiguous()
        for kind, x, codes, top, rec in ((PQ_KEY, k, kc, kt, k_rec), (PQ_VALUE, v, vc, vt, v_rec)):
            # the attention kernels run on the oracle's own records, laid out as tiles by the numpy layout reference
            # (see build_cache in test_gpu_parity.py): nothing a library kernel produced reaches the oracle
            rec_or = oracle_records(x, S, cb, bits, cbt)[0]
            rec[:, starts[b]:starts[b] + n] = rec_or
            helpers.upload_records_deep(kind, rec_or, codes, top, starts[b])
    torch.cuda.synchronize()
    return (kc, kt, vc, vt), np.array(starts, dtype=np.int64), pool, k_rec, v_rec


@pytest.mark.parametrize("bits,Hq,Hkv", [((2, 2, 2), 8, 2), ((3, 1, 1), 2, 2), ((1, 3, 2), 3, 3)])
def test_deep_attention(bits, Hq, Hkv):
    ctx, S, cb, cbt = make(bits)
    lens = [1, 64, 65, 0, 1000, 64 * 7 + 3]
    say(f"deep attention bits={bits} Hq={Hq} Hkv={Hkv} lens={lens}")
    B = len(lens)
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, bits, cbt, lens, Hkv, seed=1300)
    kc, kt, vc, vt = caches
    q = synth.queries(B, Hq, seed=1301)
    out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(Context.attn_workspace_bytes(B, Hq, Hkv, max(lens)), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    ctx.attn_decode_polar(q.to(DEV), out, kc, kt, vc, vt, torch.from_numpy(starts).to(DEV),
                          torch.tensor(lens, dtype=torch.int32, device=DEV), max(lens), helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.attention_deep(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb, bits,
                                cbt, helpers.softmax_scale())
    assert np.all(np.isfinite(got)) and np.all(got[3] == 0.0)
    per_seq = [helpers.rel_l2(got[b], ref[b]) if lens[b] else 0.0 for b in range(B)]
    say(f"  rel L2 {helpers.rel_l2(got, ref):.2e}; per sequence {['%.1e' % e for e in per_seq]}")
    assert max(per_seq) <= 2e-3


def test_deep_hybrid_attention():
    """Deep-format prefix + unquantised bf16 window, one softmax over both."""
    bits = (2, 2, 2)
    ctx, S, cb, cbt = make(bits)
    Hq, Hkv = 8, 2
    lens = [0, 0, 100, 1000, 64, 300]
    wins = [0, 5, 1, 63, 64, 130]
    cap = 130
    say(f"deep hybrid attention prefix={lens} window={wins}")
    B = len(lens)
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, bits, cbt, lens, Hkv, seed=1500)
    kc, kt, vc, vt = caches
    g = torch.Generator().manual_seed(1501)
    win_k = torch.randn((B, Hkv, cap, 128), generator=g).to(torch.bfloat16)
    win_v = torch.randn((B, Hkv, cap, 128), generator=g).to(torch.bfloat16)
    win_k[:, :, :, 7] *= 6.0
    q = synth.queries(B, Hq, seed=1502)
    out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(Context.attn_hybrid_workspace_bytes(B, Hq, Hkv, max(lens), cap), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    ctx.attn_decode_hybrid(q.to(DEV), out, kc, kt, vc, vt, torch.from_numpy(starts).to(DEV),
                           torch.tensor(lens, dtype=torch.int32, device=DEV), win_k.to(DEV), win_v.to(DEV),
                           torch.tensor(wins, dtype=torch.int32, device=DEV), max(lens), helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.attention_hybrid_deep(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32),
                                       win_k.to(torch.float64).numpy(), win_v.to(torch.float64).numpy(),
                                       np.array(wins, np.int32), S, cb, bits, cbt, helpers.softmax_scale())
    assert np.all(np.isfinite(got)) and np.all(got[0] == 0.0)
    per_seq = [helpers.rel_l2(got[b], ref[b]) for b in range(1, B)]
    say(f"  per sequence {['%.1e' % e for e in per_seq]}")
    assert max(per_seq) <= 2e-3 and per_seq[0] <= 1e-5     # sequence 1 is window only: fp32 accuracy


def test_deep_decode_step():
    bits = (2, 2, 2)
    ctx, S, cb, cbt = make(bits)
    Hq, Hkv, lens = 8, 2, [130, 64, 700]
    B = len(lens)
    say(f"deep decode step (append newest token, then attention) lens={lens}")
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, bits, cbt, [n - 1 for n in lens], Hkv, seed=1400)
    kc, kt, vc, vt = caches
    new_k = synth.kv_stream(B, Hkv, seed=1410).permute(1, 0, 2).contiguous()      # [B, Hkv, 128]
    new_v = synth.kv_stream(B, Hkv, seed=1411).permute(1, 0, 2).contiguous()
    q = synth.queries(B, Hq, seed=1412)
    slots = torch.tensor([int(starts[b]) + lens[b] - 1 for b in range(B)], dtype=torch.int64, device=DEV)
    out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(Context.attn_workspace_bytes(B, Hq, Hkv, max(lens)), dtype=torch.uint8, device=DEV)
    d_start = torch.from_numpy(starts).to(DEV)
    d_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    ctx.decode_step_polar(new_k.to(DEV), new_v.to(DEV), slots, q.to(DEV), out, kc, kt, vc, vt, d_start, d_len, max(lens),
                          helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    for b in range(B):      # the appended tokens: the library's records are held to the oracle's, which are what the oracle attends on
        for kind, x, codes, top, rec in ((PQ_KEY, new_k, kc, kt, k_rec), (PQ_VALUE, new_v, vc, vt, v_rec)):
            rec_or, psi, y = oracle_records(x[b:b + 1], S, cb, bits, cbt)
            tile0 = (int(slots[b]) // 64) * 64
            rec_gpu = export_both_ways(ctx, kind, codes, top, tile0, 64)[:, int(slots[b]) - tile0][:, None]
            check_records(rec_gpu, rec_or, psi, y, bits)
            rec[:, int(slots[b])] = rec_or[:, 0]
    ref = oracle.attention_deep(q.to(torch.float64).numpy(), k_rec, v_rec, starts, np.array(lens, np.int32), S, cb, bits,
                                cbt, helpers.softmax_scale())
    err = helpers.rel_l2(out.cpu().numpy(), ref)
    say(f"  rel L2 {err:.2e}")
    assert err <= 2e-3


@pytest.mark.parametrize("M,Hq,Hkv", [(2, 8, 2), (4, 4, 1), (1, 16, 2), (3, 2, 2)])
def test_deep_multi_query_attention(M, Hq, Hkv):
    """Several query tokens per sequence (and groups of 8 query heads) on depth-7 caches: row (b, m) is
    single-query attention over the first ctx_len - (M-1-m) cached tokens."""
    bits = (2, 2, 2)
    ctx, S, cb, cbt = make(bits)
    lens = [M, 64, 65 + M, 1000, 64 * 5 + 1]
    say(f"deep multi-query attention M={M} Hq={Hq} Hkv={Hkv} lens={lens}")
    B = len(lens)
    caches, starts, pool, k_rec, v_rec = build_cache(ctx, S, cb, bits, cbt, lens, Hkv, seed=1600 + M)
    kc, kt, vc, vt = caches
    q = synth.queries(B * M, Hq, seed=1601).reshape(B, M, Hq, 128).contiguous()
    out = torch.full((B, M, Hq, 128), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(Context.attn_mq_workspace_bytes(B, M, Hq, Hkv, max(lens)), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    ctx.attn_decode_polar_mq(q.to(DEV), out, kc, kt, vc, vt, torch.from_numpy(starts).to(DEV),
                             torch.tensor(lens, dtype=torch.int32, device=DEV), max(lens), helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    errs = []
    for m in range(M):
        lens_m = np.array([max(n - (M - 1 - m), 0) for n in lens], dtype=np.int32)
        ref = oracle.attention_deep(q[:, m].to(torch.float64).numpy(), k_rec, v_rec, starts, lens_m, S, cb, bits, cbt,
                                    helpers.softmax_scale())
        errs.append(helpers.rel_l2(got[:, m], ref))
        for b in range(B):
            if lens_m[b] == 0:
                assert np.all(got[b, m] == 0.0)
            else:
                assert helpers.rel_l2(got[b, m], ref[b]) <= 2e-3, (b, m)
    say(f"  rel L2 per query token {['%.1e' % e for e in errs]}")
