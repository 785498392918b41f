"""GPU test of pq_attn_decode_polar_static, the attention entry point that allocates nothing.

It is compared, through the C ABI, with pq_attn_decode_polar (the existing entry point whose
kernels it shares) on two calls in a row, the second with a smaller input, so that whatever the
first call left in the library's static scratch array would show in the second.  The existing entry
point is itself held to the oracle by the parity tests; here the two must agree bit for bit.
"""
import sys

import numpy as np
import pytest
import torch

from paper_2502_02617_amd import Context, PQ_KEY, PQ_VALUE, PolarQuantError, synth
from tests import helpers

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


def _batch(ctx, lens, Hq, Hkv, seed):
    starts, pool = [], 0
    for n in lens:
        starts.append(pool)
        pool += ((max(n, 1) + 63) // 64) * 64
    kc, kr = Context.alloc_cache(Hkv, pool, DEV)
    vc, vr = Context.alloc_cache(Hkv, pool, DEV)
    for t in (kc, vc):
        t.fill_(0xFF)
    for t in (kr, vr):
        t.fill_(0x7E00)
    streams = []
    for b, n in enumerate(lens):
        k = synth.kv_stream(n, Hkv, seed + 2 * b).permute(1, 0, 2).contiguous()
        v = synth.kv_stream(n, Hkv, seed + 2 * b + 1).permute(1, 0, 2).contiguous()
        ctx.encode_kv(k.to(DEV), PQ_KEY, kc, kr, dst_token0=starts[b])
        ctx.encode_kv(v.to(DEV), PQ_VALUE, vc, vr, dst_token0=starts[b])
        streams.append((k, v))
    q = synth.queries(len(lens), Hq, seed=seed)
    torch.cuda.synchronize()
    return (kc, kr, vc, vr), np.array(starts, dtype=np.int64), pool, q, streams


def _both(ctx, caches, starts, lens, q, out_dtype):
    kc, kr, vc, vr = caches
    B, Hq, _ = q.shape
    Hkv = kc.shape[0]
    max_ctx = max(lens)
    st = torch.from_numpy(starts).to(DEV)
    ln = torch.tensor(lens, dtype=torch.int32, device=DEV)
    qd = q.to(DEV)
    ws = torch.empty(Context.attn_workspace_bytes(B, Hq, Hkv, max_ctx), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    ref = torch.full((B, Hq, 128), float("nan"), dtype=out_dtype, device=DEV)
    ctx.attn_decode_polar(qd, ref, kc, kr, vc, vr, st, ln, max_ctx, helpers.softmax_scale(), ws)
    got = torch.full((B, Hq, 128), float("nan"), dtype=out_dtype, device=DEV)
    ctx.attn_decode_polar_static(qd, got, kc, kr, vc, vr, st, ln, max_ctx, helpers.softmax_scale())
    torch.cuda.synchronize()
    return got.float().cpu().numpy(), ref.float().cpu().numpy()


def test_static_scratch_entry_point_two_calls_in_a_row():
    ctx = Context(seed=0)
    ctx.prepare_device()
    # first call: a ragged batch that spans several tiles, a ragged tail and an empty sequence
    lens1 = [1500, 64, 0, 777, 2049]
    say(f"static scratch entry point, call 1: lens={lens1} Hq=8 Hkv=2")
    caches1, starts1, pool1, q1, streams1 = _batch(ctx, lens1, 8, 2, seed=900)
    got1, ref1 = _both(ctx, caches1, starts1, lens1, q1, torch.float32)
    assert np.all(np.isfinite(got1))
    assert np.array_equal(got1, ref1), "static-scratch call differs from pq_attn_decode_polar"
    assert np.all(got1[2] == 0.0)
    # second call right after it: a smaller input (fewer sequences, shorter contexts, other head counts)
    lens2 = [130, 5]
    say(f"static scratch entry point, call 2 (smaller): lens={lens2} Hq=4 Hkv=1")
    caches2, starts2, pool2, q2, _ = _batch(ctx, lens2, 4, 1, seed=901)
    got2, ref2 = _both(ctx, caches2, starts2, lens2, q2, torch.bfloat16)
    assert np.all(np.isfinite(got2))
    assert np.array_equal(got2, ref2), "second (smaller) static-scratch call differs from pq_attn_decode_polar"


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    ctx = Context(seed=0)
    fresh = Context(seed=1)
    ctx.prepare_device()
    B, Hq, Hkv, max_ctx = 2048, 32, 8, 4096
    assert Context.attn_workspace_bytes(B, Hq, Hkv, max_ctx) > Context.static_scratch_bytes()
    kc, kr = Context.alloc_cache(1, 64, DEV)
    q = torch.zeros((B, Hq, 128), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros_like(q)
    st = torch.zeros(B, dtype=torch.int64, device=DEV)
    ln = torch.zeros(B, dtype=torch.int32, device=DEV)
    say("static scratch entry point: a problem beyond the array is refused (PQ_ESCRATCH), nothing is launched")
    with pytest.raises(PolarQuantError, match="PQ_ESCRATCH"):
        ctx.attn_decode_polar_static(q, out, kc, kr, kc, kr, st, ln, max_ctx, helpers.softmax_scale())
    say("static scratch entry point: a context whose constants are not on the device is refused (PQ_ENOTREADY)")
    with pytest.raises(PolarQuantError, match="PQ_ENOTREADY"):
        fresh.attn_decode_polar_static(q[:1, :4], out[:1, :4], kc, kr, kc, kr, st[:1], ln[:1], 64, helpers.softmax_scale())
    torch.cuda.synchronize()
