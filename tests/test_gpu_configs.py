"""GPU parity at the full sizes of the benchmark configurations, on sampled outputs.

The launch configurations are the ones bench.py times.  Inputs are drawn on the GPU
with the seeded recipes of synth.py (same recipe as the CPU draws, other random
stream) and the sampled parts are copied to the host for the fp64 oracle, which
encodes and attends on its own.
"""
import math
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2502_02617_amd import Context, PQ_KEY, PQ_VALUE, synth
from tests import helpers

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


def run_attention_case(ctx, S, cb, lens, sample_pairs, seed, append=False):
    """Builds the cache of a whole batch on the GPU, runs pq_attn_decode_polar for all rows and
    checks the sampled (sequence, kv head) pairs against the oracle."""
    B = len(lens)
    starts, pool = [], 0
    for n in lens:
        starts.append(pool)
        pool += ((n + 63) // 64) * 64 + 64
    kc, kr = Context.alloc_cache(HKV, pool, DEV)
    vc, vr = Context.alloc_cache(HKV, pool, DEV)
    for t in (kc, kr, vc, vr):
        t.zero_()
    wanted = {}
    for b, hk in sample_pairs:
        wanted.setdefault(b, []).append(hk)
    kept = {}
    for b, n in enumerate(lens):
        k = synth.kv_stream(n, HKV, seed=seed + 2 * b, device=DEV)
        v = synth.kv_stream(n, HKV, seed=seed + 2 * b + 1, device=DEV)
        n_bulk = n - 1 if append else n
        encode_stream(ctx, k[:, :n_bulk], PQ_KEY, kc, kr, starts[b])
        encode_stream(ctx, v[:, :n_bulk], PQ_VALUE, vc, vr, starts[b])
        if append:
            kept.setdefault("new_k", []).append(k[:, n - 1])
            kept.setdefault("new_v", []).append(v[:, n - 1])
        for hk in wanted.get(b, []):
            kept[(b, hk)] = (k[hk:hk + 1].clone(), v[hk:hk + 1].clone())
        del k, v
    seq_start = torch.tensor(starts, dtype=torch.int64, device=DEV)
    ctx_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    if append:  # decode-time order: append the newest token of every sequence, then attend
        newest = seq_start + ctx_len.to(torch.int64) - 1
        ctx.append_kv(torch.stack(kept["new_k"]).contiguous(), PQ_KEY, kc, kr, newest)
        ctx.append_kv(torch.stack(kept["new_v"]).contiguous(), PQ_VALUE, vc, vr, newest)
    q = synth.queries(B, HQ, seed=seed + 999, device=DEV)
    out = torch.empty((B, HQ, 128), dtype=torch.float32, device=DEV)
    max_ctx = max(lens)
    ws = torch.empty(Context.attn_workspace_bytes(B, HQ, HKV, max_ctx), dtype=torch.uint8, device=DEV)
    ctx.attn_decode_polar(q, out, kc, kr, vc, vr, seq_start, ctx_len, max_ctx, SCALE, ws)
    torch.cuda.synchronize()
    got_all = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got_all))
    got, ref = [], []
    for b, hk in sample_pairs:
        k, v = kept[(b, hk)]
        k_rec = oracle_encode_heads(k, S, cb)[0]
        v_rec = oracle_encode_heads(v, S, cb)[0]
        qs = q[b:b + 1, 4 * hk:4 * hk + 4].cpu().to(torch.float64).numpy()
        r = oracle.attention(qs, k_rec, v_rec, np.array([0], np.int64), np.array([lens[b]], np.int32), S, cb, SCALE)
        ref.append(r[0])
        got.append(got_all[b, 4 * hk:4 * hk + 4])
    got, ref = np.stack(got), np.stack(ref)
    err = helpers.rel_l2(got, ref)
    per_pair = [helpers.rel_l2(g, r) for g, r in zip(got, ref)]
    say(f"  sampled pairs {sample_pairs}: rel L2 {err:.2e}; per pair {['%.1e' % e for e in per_pair]}")
    return err


def test_config2_decode_32k(env):
    ctx, S, cb = env
    say("config 2: batch 16, 32768-token context, sampled (sequence, kv head) pairs")
    pairs = [(0, 0), (3, 5), (7, 2), (9, 7), (12, 4), (15, 1), (5, 3), (10, 6)]
    err = run_attention_case(ctx, S, cb, [32768] * 16, pairs, seed=2000)
    assert err <= 2e-3


def test_config3_long_context_128k(env):
    ctx, S, cb = env
    say("config 3: batch 4, 131072-token context")
    pairs = [(0, 0), (1, 3), (2, 6), (3, 7)]
    err = run_attention_case(ctx, S, cb, [131072] * 4, pairs, seed=3000)
    assert err <= 2e-3


def test_config4_ragged_serving_step(env):
    ctx, S, cb = env
    lens = [int(n) for n in synth.ragged_lengths(64, 1024, 65536, seed=4)]
    say(f"config 4: 64 ragged sequences, lengths {min(lens)}..{max(lens)}, append then attend")
    order = np.argsort(lens)
    picks = [int(order[0]), int(order[-1]), int(order[len(order) // 2]), int(order[5]), int(order[-5]), 17]
    pairs = [(b, (3 * i) % HKV) for i, b in enumerate(picks)]
    err = run_attention_case(ctx, S, cb, lens, pairs, seed=4000, append=True)
    assert err <= 2e-3
