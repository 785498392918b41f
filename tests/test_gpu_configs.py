"""GPU parity at the full sizes of the benchmark configurations.

The launch configurations are the ones bench.py times.  Inputs are drawn on the GPU
with the seeded recipes of synth.py (same recipe as the CPU draws, other random
stream) and copied to the host for the fp64 oracle, which encodes and attends on its own:
config 2 and config 3 on every output row, config 4 (one layer) on every sequence with one of
its kv heads, so that every sequence and every kv head is covered.
"""
import math
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2502_02617_amd import Context, PQ_KEY, PQ_VALUE, synth
from tests import helpers, layout_ref

pytestmark = pytest.mark.gpu
DEV = "cuda"
HQ, HKV = 32, 8
SCALE = 1.0 / math.sqrt(128.0)


def say(msg):
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def env():
    return Context(seed=0), oracle.preconditioner(0), oracle.default_codebooks()


def oracle_encode_heads(x_dev, S, cb):
    """x_dev [H, T, 128] bf16 on the GPU -> records [H, T, 62] (+ exact angles, rotated vectors)."""
    H, T, _ = x_dev.shape
    x = x_dev.cpu().to(torch.float64).numpy().reshape(H * T, 128)
    rec, psi, y = oracle.encode(x, S, cb, want_psi=True, want_y=True)
    return rec.reshape(H, T, 62), psi.reshape(H, T, 120), y.reshape(H, T, 128)


def encode_stream(ctx, x, kind, codes, radii, dst0):
    """x [H, T, 128] head-major on the GPU, read through strides."""
    ctx.encode_kv(x, kind, codes, radii, dst_token0=dst0, ld_token=x.stride(1), ld_head=x.stride(0),
                  n_tokens=x.shape[1], n_heads=x.shape[0])


# ---------------------------------------------------------------------------
# config 1: single-layer KV encode, 8 KV heads x 32768 tokens, bf16 with outlier channels
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kind", [PQ_KEY, PQ_VALUE])
def test_config1_encode_all_vectors(env, kind):
    ctx, S, cb = env
    T = 32768
    say(f"config 1 encode kind={kind}: {HKV} heads x {T} tokens")
    x = synth.kv_stream(T, HKV, seed=1 + kind, device=DEV)
    codes, radii = Context.alloc_cache(HKV, T, DEV)
    encode_stream(ctx, x, kind, codes, radii, 0)
    rec = torch.empty((HKV, T, 62), dtype=torch.uint8, device=DEV)
    ctx.export_canonical(kind, codes, radii, 0, T, rec)
    torch.cuda.synchronize()
    rec_or, psi, y = oracle_encode_heads(x, S, cb)
    st, rg, ro = helpers.check_codes(rec.cpu().numpy().reshape(-1, 62), rec_or.reshape(-1, 62), psi.reshape(-1, 120))
    st.update(helpers.check_radii(rg, ro, y.reshape(-1, 128)))
    say(f"  {st}")
    # DeQuant of the whole stream against the oracle's DeQuant of its own records
    out = torch.empty((T, HKV, 128), dtype=torch.float32, device=DEV)
    ctx.decode_kv(kind, codes, radii, 0, T, out, rotated=False)
    torch.cuda.synchronize()
    ref = oracle.decode(rec_or.reshape(-1, 62), S, cb).reshape(HKV, T, 128)
    err = helpers.rel_l2(out.cpu().numpy().transpose(1, 0, 2), ref)
    say(f"  DeQuant rel L2 {err:.2e}")
    assert err <= 1e-3


def row_errors(got, ref):
    """Error of every output row relative to its own norm or to the root-mean-square row norm of the reference,
    whichever is larger (a row whose output nearly cancels has a small norm of its own but the same absolute
    error as its neighbours)."""
    rms = math.sqrt(float(np.mean(np.sum(ref * ref, axis=-1))))
    return np.sqrt(np.sum((got - ref) ** 2, axis=-1)) / np.maximum(np.sqrt(np.sum(ref * ref, axis=-1)), rms)


def run_attention_case(ctx, S, cb, lens, heads_of, seed, step=False):
    """Builds the cache of a whole batch on the GPU with the library's encoder, runs attention for all rows in the
    launch configuration bench.py times, and checks the (sequence, kv head) pairs named by heads_of(b) against the
    oracle, which encodes the same inputs and attends on its own records.
    step=False: pq_attn_decode_polar, fp32 output.
    step=True:  the newest token of every sequence goes in through pq_decode_step_polar (append + attention in one
                call, bf16 output: what bench.py times), then pq_attn_decode_polar with fp32 output runs on the
                same cache; both are checked.
    Returns {label: (rel L2 over the compared rows, worst row error, rel L2 of the oracle's result rounded to the output format)}."""
    B = len(lens)
    starts, pool = [], 0
    for n in lens:
        starts.append(pool)
        pool += ((n + 63) // 64) * 64 + 64
    kc, kr = Context.alloc_cache(HKV, pool, DEV)
    vc, vr = Context.alloc_cache(HKV, pool, DEV)
    for t in (kc, kr, vc, vr):
        t.zero_()
    q = synth.queries(B, HQ, seed=seed + 999, device=DEV)
    q_host = q.cpu().to(torch.float64).numpy()
    new_k, new_v, ref, where = [], [], [], []
    for b, n in enumerate(lens):
        k = synth.kv_stream(n, HKV, seed=seed + 2 * b, device=DEV)
        v = synth.kv_stream(n, HKV, seed=seed + 2 * b + 1, device=DEV)
        n_bulk = n - 1 if step else n
        encode_stream(ctx, k[:, :n_bulk], PQ_KEY, kc, kr, starts[b])
        encode_stream(ctx, v[:, :n_bulk], PQ_VALUE, vc, vr, starts[b])
        if step:
            new_k.append(k[:, n - 1])
            new_v.append(v[:, n - 1])
        heads = list(heads_of(b))
        if heads:   # the oracle's side of this sequence: its own records of the same inputs, then Eq. 5
            k_rec = oracle_encode_heads(k[heads], S, cb)[0]
            v_rec = oracle_encode_heads(v[heads], S, cb)[0]
            qs = np.concatenate([q_host[b:b + 1, 4 * hk:4 * hk + 4] for hk in heads], axis=1)
            r = oracle.attention(qs, k_rec, v_rec, np.array([0], np.int64), np.array([n], np.int32), S, cb, SCALE)
            for i, hk in enumerate(heads):
                ref.append(r[0, 4 * i:4 * i + 4])
                where.append((b, hk))
        del k, v
    ref = np.stack(ref)
    seq_start = torch.tensor(starts, dtype=torch.int64, device=DEV)
    ctx_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    max_ctx = max(lens)
    ws = torch.empty(Context.attn_workspace_bytes(B, HQ, HKV, max_ctx), dtype=torch.uint8, device=DEV)
    outs = {}
    if step:  # decode-time order: the newest token of every sequence is appended, then attended to
        newest = seq_start + ctx_len.to(torch.int64) - 1
        out_b = torch.empty((B, HQ, 128), dtype=torch.bfloat16, device=DEV)
        ctx.decode_step_polar(torch.stack(new_k).contiguous(), torch.stack(new_v).contiguous(), newest, q, out_b,
                              kc, kr, vc, vr, seq_start, ctx_len, max_ctx, SCALE, ws)
        outs["pq_decode_step_polar bf16"] = out_b
    out = torch.empty((B, HQ, 128), dtype=torch.float32, device=DEV)
    ctx.attn_decode_polar(q, out, kc, kr, vc, vr, seq_start, ctx_len, max_ctx, SCALE, ws)
    outs["pq_attn_decode_polar fp32"] = out
    torch.cuda.synchronize()
    result = {}
    for label, o in outs.items():
        got_all = o.float().cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(got_all))
        got = np.stack([got_all[b, 4 * hk:4 * hk + 4] for b, hk in where])
        err = helpers.rel_l2(got, ref)
        rows = row_errors(got.reshape(-1, 128), ref.reshape(-1, 128))
        say(f"  {label}: {len(where)} (sequence, kv head) pairs = {rows.size} rows: rel L2 {err:.2e}; "
            f"worst row {rows.max():.2e}")
        # what rounding the oracle's own result to the output format costs (zero for fp32 output)
        fmt = helpers.rel_l2(torch.from_numpy(ref).to(o.dtype).double().numpy(), ref)
        result[label] = (err, float(rows.max()), fmt)
    return result


# Bounds.  Attention: 2e-3 relative L2 over the compared rows (bf16 inputs, fp32 output).  A bf16 output is the same
# numbers rounded to 8 significant bits, which by itself costs 1.7e-3 .. 2.0e-3 relative L2 (measured on the oracle's
# own result), so for bf16 output the format's rounding is added in quadrature; config 2, the configuration the
# benchmark times, is additionally held to the flat 2e-3 with bf16 output.
# Single rows are heavy-tailed -- a row dominated by one or two tokens carries those tokens' quantisation and rounding
# errors undiluted, and the encoder may code an angle on a cell boundary either way -- so the per-row limit is a
# detector of gross errors (a piece of a stream attended twice or not at all moves a row by far more): ten times the
# aggregate tolerance.  Measured worst rows: 2.8e-3 (fp32 output), 3.9e-3 (bf16 output) of the 512 of config 2.
ATTN_TOL, ROW_TOL = 2e-3, 2e-2


def check_case(result, flat_bf16=False):
    for label, (err, worst, fmt) in result.items():
        bound = ATTN_TOL if flat_bf16 else math.sqrt(ATTN_TOL ** 2 + fmt ** 2)
        assert err <= bound, (label, err, bound)
        assert worst <= ROW_TOL, (label, worst)


def test_config2_decode_32k(env):
    ctx, S, cb = env
    say("config 2: batch 16, 32768-token context, all 512 output rows, decode step (bf16) and attention (fp32)")
    check_case(run_attention_case(ctx, S, cb, [32768] * 16, lambda b: range(HKV), seed=2000, step=True), flat_bf16=True)


def test_config3_long_context_128k(env):
    ctx, S, cb = env
    say("config 3: batch 4, 131072-token context, all 128 output rows")
    check_case(run_attention_case(ctx, S, cb, [131072] * 4, lambda b: range(HKV), seed=3000))


def test_config4_ragged_serving_step(env):
    ctx, S, cb = env
    lens = [int(n) for n in synth.ragged_lengths(64, 1024, 65536, seed=4)]
    say(f"config 4: 64 ragged sequences, lengths {min(lens)}..{max(lens)}, decode step (append, then attend); "
        "every sequence with one kv head, every kv head eight times")
    check_case(run_attention_case(ctx, S, cb, lens, lambda b: [(b + b // HKV) % HKV], seed=4000, step=True))


def test_one_sequence_of_a_million_tokens(env):
    """A single sequence of 1000003 tokens (ragged last tile): all wavefronts of the launch work on the eight streams
    of one sequence, every stream is cut into about 500 pieces that the combine step merges, and the newest token is
    appended at the end of the longest cache any test builds.  Two of the kv heads against the oracle."""
    ctx, S, cb = env
    n = 1000003
    say(f"one sequence of {n} tokens, decode step (append, then attend); kv heads 0 and 7 against the oracle")
    check_case(run_attention_case(ctx, S, cb, [n], lambda b: [0, HKV - 1], seed=5000, step=True))


# ---------------------------------------------------------------------------
# a cache whose code planes are larger than 4 GiB: sequences that live beyond the 2^32-byte mark
# ---------------------------------------------------------------------------
def test_cache_planes_beyond_four_gib():
    """8 kv heads x 190000 tiles: 4.47 GB of key codes (and as many of value codes), so the tiles of the last head
    near the end of the pool start more than 2^32 bytes into the buffer.  Bulk encode, append, export and attention on
    two short sequences placed there, against the oracle: every address on the way has to be formed in 64 bits."""
    ctx = Context(seed=0)
    S, cb = oracle.preconditioner(0), oracle.default_codebooks()
    tiles = 190000
    pool = tiles * 64
    kc, kr = Context.alloc_cache(HKV, pool, DEV)
    vc, vr = Context.alloc_cache(HKV, pool, DEV)
    assert kc.numel() > (1 << 32) and (HKV - 1) * tiles * 2944 + (tiles - 1200) * 2944 > (1 << 32)
    lens = [100, 300]
    starts = [(tiles - 1000) * 64, (tiles - 500) * 64]
    say(f"cache planes of {kc.numel() / 1e9:.2f} GB: sequences of {lens} tokens at tiles {[s0 // 64 for s0 in starts]}")
    k_rec = {}
    v_rec = {}
    n_ties = 0
    for b, (s0, n) in enumerate(zip(starts, lens)):
        k = synth.kv_stream(n + 1, HKV, 4200 + 2 * b).permute(1, 0, 2).contiguous()   # [n + 1, HKV, 128]; the last one is appended
        v = synth.kv_stream(n + 1, HKV, 4201 + 2 * b).permute(1, 0, 2).contiguous()
        for t in (kc, kr, vc, vr):
            t[:, s0 // 64 : s0 // 64 + (n + 64) // 64 + 1].zero_()
        ctx.encode_kv_pair(k[:n].to(DEV), v[:n].to(DEV), kc, kr, vc, vr, dst_token0=s0)
        dst = torch.tensor([s0 + n], dtype=torch.int64, device=DEV)
        ctx.append_kv_pair(k[n:].to(DEV), v[n:].to(DEV), kc, kr, vc, vr, dst)
        torch.cuda.synchronize()
        for kind, x, codes, radii, store in ((PQ_KEY, k, kc, kr, k_rec), (PQ_VALUE, v, vc, vr, v_rec)):
            rec = torch.empty((HKV, n + 1, 62), dtype=torch.uint8, device=DEV)
            ctx.export_canonical(kind, codes, radii, s0, n + 1, rec)
            torch.cuda.synchronize()
            rec = rec.cpu().numpy()
            # the same tiles read by the numpy layout reference (only the slices in question leave the device)
            T = (n + 1 + 63) // 64
            for h in (0, HKV - 1):
                c_h = codes[h, s0 // 64 : s0 // 64 + T].cpu().numpy()
                r_h = radii[h, s0 // 64 : s0 // 64 + T].cpu().numpy().view(np.uint16)
                assert np.array_equal(rec[h], layout_ref.tiles_to_canonical(kind, c_h, r_h, n + 1))
            xs = x.permute(1, 0, 2).contiguous().to(torch.float64).numpy().reshape(HKV * (n + 1), 128)
            rec_or, psi, y = oracle.encode(xs, S, cb, want_psi=True, want_y=True)
            st, rg, ro = helpers.check_codes(rec.reshape(-1, 62), rec_or, psi, enforce_rate=False)
            helpers.check_radii(rg, ro, y, enforce_rate=False)
            n_ties += st["code_mismatches"]
            store[b] = rec_or.reshape(HKV, n + 1, 62)
            # attention below runs on the oracle's own records
            helpers.upload_records(kind, store[b], codes, radii, s0)
    assert n_ties <= 2
    B, Hq = len(lens), 32
    q = synth.queries(B, Hq, seed=4210)
    ctx_len = [n + 1 for n in lens]
    out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(Context.attn_workspace_bytes(B, Hq, HKV, max(ctx_len)), dtype=torch.uint8, device=DEV)
    ctx.attn_decode_polar(q.to(DEV), out, kc, kr, vc, vr, torch.tensor(starts, dtype=torch.int64, device=DEV),
                          torch.tensor(ctx_len, dtype=torch.int32, device=DEV), max(ctx_len), helpers.softmax_scale(), ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    # the oracle sees a small pool holding just the two sequences
    small_starts, at = [], 0
    for n in ctx_len:
        small_starts.append(at)
        at += ((n + 63) // 64) * 64
    kk = np.zeros((HKV, at, 62), dtype=np.uint8)
    vv = np.zeros((HKV, at, 62), dtype=np.uint8)
    for b, n in enumerate(ctx_len):
        kk[:, small_starts[b] : small_starts[b] + n] = k_rec[b]
        vv[:, small_starts[b] : small_starts[b] + n] = v_rec[b]
    ref = oracle.attention(q.to(torch.float64).numpy(), kk, vv, np.array(small_starts, np.int64), np.array(ctx_len, np.int32),
                           S, cb, helpers.softmax_scale())
    err = helpers.rel_l2(got, ref)
    say(f"  appended + encoded records: {n_ties} ties; attention rel L2 {err:.2e}")
    assert np.all(np.isfinite(got)) and err <= ATTN_TOL
    del kc, kr, vc, vr
    torch.cuda.empty_cache()
