#!/usr/bin/env python3
"""Benchmark of the PolarQuant hot path on one MI355X.

Workload (benchmark configs[2], the one the headline metric is quoted on):
GQA decode attention on a polar-quantised KV cache, batch 16, 32 query heads /
8 KV heads, 32768-token context, d = 128, one bf16 query per sequence.

One step = one pass of the whole hot path for one decode iteration:
  pq_decode_step_polar  = pq_append_kv_pair + pq_attn_decode_polar (same results, one launch fewer):
     append             encode the newest key and value of every sequence (rotate, polar, quantise, pack)
     attention          rotate q, attention on the packed codes, combine, un-rotate
The value is the cache bandwidth the whole step sustains: 124 bytes per cached
(token, kv head) -- one 62-byte key record and one 62-byte value record --
divided by the step time.  Three distinct caches are used in rotation so that
consecutive steps cannot be served from the 256 MB last-level cache.

Also reported: the roofline line of the dominant kernel (HIP events recorded
around it on the launch stream during the timed steps), bulk-encode throughput
on benchmark configs[1] (8 KV heads x 32768 tokens, keys and values), the
decode step on configs[3] (batch 4 x 131072 tokens) and configs[4] (64 ragged
sequences, 32 layers per step), the widened entry points (hybrid, several
query tokens, full recursion depth), and the fp64 CPU oracle timed on a
bounded sample of the same workload.

The default warm-up is 100 steps (16 ms of GPU work): after the idle time of
the set-up the chip needs some milliseconds of load to reach its steady
clock, and the first steps run about 4 % slower than the rest.
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
B, HQ, HKV, CTX, D = 16, 32, 8, 32768, 128
N_CACHES = 3
BYTES_PER_TOKEN_HEAD = 124  # 62-byte key record + 62-byte value record
PROFILE_FILE = os.path.join(ROOT, "profiles", "attn_partial_cfg2_counters.txt")
# Secondary bound of the dominant kernel: vector-ALU issue, as a plain instruction count against one 64-lane vector
# instruction per SIMD every 4 cycles: 256 CUs x 4 SIMDs x 2.4 GHz / 4 = 614.4 G wavefront instructions/s.  That is
# the measured rate of three-operand integer, packed binary16 and conversion instructions; plain fp32 instructions and
# shifts issue every 2 cycles and a matrix instruction (counted as one here) holds the SIMD for 8 or 16, so the
# fraction is an indication, not a bound met instruction by instruction.
VALU_PEAK_GINSTR = 256 * 4 * 2.4 / 4.0


def profile_figures():
    """Counter figures of the dominant kernel on this workload, from the tracked rocprofv3 summary (lines
    `name = value` under its "figures read by bench.py" heading; the file names the commit they were taken on).
    They come from separate profiling runs of this same script: HBM bytes per launch (FETCH_SIZE / WRITE_SIZE scaled
    by a plain copy of known size) and executed vector instructions per launch (SQ_INSTS_VALU).  {} if absent."""
    out = {}
    try:
        with open(PROFILE_FILE) as f:
            for line in f:
                parts = line.split("=")
                if len(parts) == 2 and parts[0].strip().replace("_", "").isalnum() and " " not in parts[0].strip():
                    out[parts[0].strip()] = parts[1].strip()
    except OSError:
        pass
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--encode-steps", type=int, default=60)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-seqs", type=int, default=16)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2502_02617_amd import Context, PQ_KEY, PQ_VALUE, profile_begin, profile_end, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda"
    ctx = Context(seed=0)
    scale = 1.0 / math.sqrt(D)
    pool_per_seq = CTX + 64  # every sequence starts on a tile boundary, one spare tile
    pool = B * pool_per_seq
    seq_start = torch.arange(B, dtype=torch.int64, device=dev) * pool_per_seq
    ctx_len = torch.full((B,), CTX, dtype=torch.int32, device=dev)
    newest_slot = seq_start + (CTX - 1)

    # ---- build the caches with the bulk encoder ----
    caches = []
    enc_inputs = []  # (k, v, first slot) of three sequences of cache 0, re-encoded in the encode measurement
    kept = {}  # sequences of cache 0 kept on the host for the CPU baseline
    t_setup = time.time()
    for c in range(N_CACHES):
        kc, kr = Context.alloc_cache(HKV, pool, dev)
        vc, vr = Context.alloc_cache(HKV, pool, dev)
        for t in (kc, kr, vc, vr):
            t.zero_()
        for b in range(B):
            k = synth.kv_stream(CTX, HKV, seed=1000 * c + 2 * b, device=dev)      # [HKV, CTX, 128] bf16
            v = synth.kv_stream(CTX, HKV, seed=1000 * c + 2 * b + 1, device=dev)
            ctx.encode_kv(k, PQ_KEY, kc, kr, dst_token0=b * pool_per_seq, ld_token=k.stride(1), ld_head=k.stride(0),
                          n_tokens=CTX, n_heads=HKV)
            ctx.encode_kv(v, PQ_VALUE, vc, vr, dst_token0=b * pool_per_seq, ld_token=v.stride(1), ld_head=v.stride(0),
                          n_tokens=CTX, n_heads=HKV)
            if c == 0 and b < 3:
                enc_inputs.append((k, v, b * pool_per_seq))
            if c == 0 and b < args.cpu_sample_seqs and not args.no_cpu_baseline:
                kept[b] = (k.cpu(), v.cpu())
            del k, v
        caches.append((kc, kr, vc, vr))
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    q = synth.queries(B, HQ, seed=7, device=dev)
    new_k = synth.kv_stream(B, HKV, seed=8, device=dev).permute(1, 0, 2).contiguous()  # [B, HKV, 128]
    new_v = synth.kv_stream(B, HKV, seed=9, device=dev).permute(1, 0, 2).contiguous()
    out = torch.empty((B, HQ, D), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(Context.attn_workspace_bytes(B, HQ, HKV, CTX), dtype=torch.uint8, device=dev)

    def step(i):
        kc, kr, vc, vr = caches[i % N_CACHES]
        ctx.decode_step_polar(new_k, new_v, newest_slot, q, out, kc, kr, vc, vr, seq_start, ctx_len, CTX, scale, ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # the partial kernel of every fourth step is bracketed by HIP events (the records cost ~2 us of stream
    # time each; timing every step would slow the timed region by 2-3 %)
    profile_begin(args.steps + 1, every=4)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = profile_end()

    ms_per_step = 1e3 * elapsed / args.steps
    step_bytes = BYTES_PER_TOKEN_HEAD * B * HKV * CTX
    value = step_bytes / (elapsed / args.steps) / 1e9
    kern_ms = prof["attn_ms"] / max(prof["attn_launches"], 1)
    achieved = step_bytes / (kern_ms * 1e-3) / 1e9 if kern_ms > 0 else 0.0

    # ---- encode line (configs[1]: 8 KV heads x 32768 tokens, keys + values = 16 vectors per token):
    # the same three sequences are encoded again into their own slots of cache 0 (same bytes as
    # before), keys and values in one launch per step (pq_encode_kv_pair), timed by HIP events on its stream
    kc, kr, vc, vr = caches[0]

    def encode_step(i):
        k, v, slot0 = enc_inputs[i % len(enc_inputs)]
        ctx.encode_kv_pair(k, v, kc, kr, vc, vr, dst_token0=slot0, ld_token=k.stride(1), ld_head=k.stride(0),
                           n_tokens=CTX, n_heads=HKV)

    for i in range(args.warmup):
        encode_step(i)
    torch.cuda.synchronize()
    profile_begin(args.encode_steps + 2)
    for i in range(args.encode_steps):
        encode_step(i)
    torch.cuda.synchronize()
    pr = profile_end()
    encode_ms, encode_tokens = pr["encode_ms"], CTX * args.encode_steps
    enc_mtok = encode_tokens / (encode_ms * 1e-3) / 1e6 if encode_ms > 0 else 0.0
    enc_bytes_per_token = 16 * (256 + 62)
    enc_gbs = enc_mtok * 1e6 * enc_bytes_per_token / 1e9

    # ---- the same encode loop with a randomised Hadamard preconditioner (one exact bf16 term of S
    # instead of three in the rotation), into a scratch cache
    ctx_h = Context(seed=0, hadamard=True)
    hk_c, hk_r = Context.alloc_cache(HKV, len(enc_inputs) * pool_per_seq, dev)
    hv_c, hv_r = Context.alloc_cache(HKV, len(enc_inputs) * pool_per_seq, dev)

    def encode_step_h(i):
        k, v, _ = enc_inputs[i % len(enc_inputs)]
        slot0 = (i % len(enc_inputs)) * pool_per_seq
        ctx_h.encode_kv_pair(k, v, hk_c, hk_r, hv_c, hv_r, dst_token0=slot0, ld_token=k.stride(1), ld_head=k.stride(0),
                             n_tokens=CTX, n_heads=HKV)

    for i in range(args.warmup):
        encode_step_h(i)
    torch.cuda.synchronize()
    profile_begin(2 * args.encode_steps + 2)
    for i in range(args.encode_steps):
        encode_step_h(i)
    torch.cuda.synchronize()
    pr_h = profile_end()
    enc_h_mtok = CTX * args.encode_steps / (pr_h["encode_ms"] * 1e-3) / 1e6 if pr_h["encode_ms"] > 0 else 0.0
    del hk_c, hk_r, hv_c, hv_r

    # ---- online codebook fit (Section 4.1): the GPU half of pq_fit_codebooks -- rotate, polar transform, count
    # every angle -- over the keys of one configs[1] sequence (8 kv heads x 32768 tokens = 262144 vectors)
    fit_ws = torch.empty(Context.fit_workspace_bytes(), dtype=torch.uint8, device=dev)
    fit_x = enc_inputs[0][0].permute(1, 0, 2)  # [tokens, heads, 128] view of the [heads, tokens, 128] stream
    for i in range(3):
        ctx.fit_count_angles(fit_x, fit_ws)
    torch.cuda.synchronize()
    fit_reps = max(args.encode_steps // 4, 2)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for i in range(fit_reps):
        ctx.fit_count_angles(fit_x, fit_ws)
    ev1.record()
    torch.cuda.synchronize()
    fit_ms = ev0.elapsed_time(ev1) / fit_reps
    fit_vectors = fit_x.shape[0] * fit_x.shape[1]
    t0 = time.perf_counter()
    ctx.fit_cluster(fit_ws.cpu().numpy().view(np.uint32), 10)
    fit_host_ms = 1e3 * (time.perf_counter() - t0)
    del fit_ws

    # ---- general format (other bit widths / recursion depths; the plain, untuned path): encode of 65536 key
    # vectors and attention of 4 sequences x 2048 tokens at depth 5, bits 4/2/2/2/2 (55 bytes per vector)
    from paper_2502_02617_amd import GeneralFormat, general_attn_decode, general_encode
    gfmt = GeneralFormat(5, [4, 2, 2, 2, 2])
    gcb = gfmt.codebooks()
    g_n, g_B, g_ctx, g_hq, g_hkv = 65536, 4, 2048, 8, 2
    gx = enc_inputs[0][0].reshape(-1, D)[:g_n]
    grec = torch.empty((g_n, gfmt.record_bytes()), dtype=torch.uint8, device=dev)
    general_encode(ctx, gfmt, gcb, gx, grec)
    torch.cuda.synchronize()
    ev0.record()
    general_encode(ctx, gfmt, gcb, gx, grec)
    ev1.record()
    torch.cuda.synchronize()
    g_enc_ms = ev0.elapsed_time(ev1)
    gk = grec[:g_hkv * g_B * g_ctx].reshape(g_hkv, g_B * g_ctx, -1)
    gv = grec[g_hkv * g_B * g_ctx:2 * g_hkv * g_B * g_ctx].reshape(g_hkv, g_B * g_ctx, -1)
    g_start = torch.arange(g_B, dtype=torch.int64, device=dev) * g_ctx
    g_len = torch.full((g_B,), g_ctx, dtype=torch.int32, device=dev)
    g_out = torch.empty((g_B, g_hq, D), dtype=torch.float32, device=dev)
    general_attn_decode(ctx, gfmt, gcb, q[:g_B, :g_hq].contiguous(), g_out, gk, gv, g_start, g_len, scale)
    torch.cuda.synchronize()
    ev0.record()
    general_attn_decode(ctx, gfmt, gcb, q[:g_B, :g_hq].contiguous(), g_out, gk, gv, g_start, g_len, scale)
    ev1.record()
    torch.cuda.synchronize()
    g_attn_ms = ev0.elapsed_time(ev1)
    del grec

    # ---- hybrid line: the same quantised 32k-token prefix plus a bf16 window of 256 recent tokens per
    # sequence (the keys and values of the generation stage kept in 16 bits), pq_attn_decode_hybrid
    WIN = 256
    win_k = synth.kv_stream(B * WIN, HKV, seed=11, device=dev).reshape(HKV, B, WIN, D).permute(1, 0, 2, 3).contiguous()
    win_v = synth.kv_stream(B * WIN, HKV, seed=12, device=dev).reshape(HKV, B, WIN, D).permute(1, 0, 2, 3).contiguous()
    win_len = torch.full((B,), WIN, dtype=torch.int32, device=dev)
    ws_h = torch.empty(Context.attn_hybrid_workspace_bytes(B, HQ, HKV, CTX, WIN), dtype=torch.uint8, device=dev)

    def hybrid_step(i):
        kc_, kr_, vc_, vr_ = caches[i % N_CACHES]
        ctx.attn_decode_hybrid(q, out, kc_, kr_, vc_, vr_, seq_start, ctx_len, win_k, win_v, win_len, CTX, scale, ws_h)

    for i in range(args.warmup):
        hybrid_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        hybrid_step(i)
    torch.cuda.synchronize()
    hybrid_ms = 1e3 * (time.perf_counter() - t0) / args.steps
    hybrid_bytes = step_bytes + 2 * 2 * D * B * HKV * WIN   # + bf16 keys and values of the window

    # ---- multi-query line: M newest tokens of every sequence query the same cache in one pass
    # (pq_attn_decode_polar_mq); the packed tile is expanded once for all M * (Hq/Hkv) columns
    mq = {}
    for M in (2, 4):
        q_m = synth.queries(B * M, HQ, seed=13, device=dev).reshape(B, M, HQ, D).contiguous()
        out_m = torch.empty((B, M, HQ, D), dtype=torch.bfloat16, device=dev)
        ws_m = torch.empty(Context.attn_mq_workspace_bytes(B, M, HQ, HKV, CTX), dtype=torch.uint8, device=dev)

        def mq_step(i):
            kc_, kr_, vc_, vr_ = caches[i % N_CACHES]
            ctx.attn_decode_polar_mq(q_m, out_m, kc_, kr_, vc_, vr_, seq_start, ctx_len, CTX, scale, ws_m)

        for i in range(args.warmup):
            mq_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            mq_step(i)
        torch.cuda.synchronize()
        mq_ms = 1e3 * (time.perf_counter() - t0) / args.steps
        mq[f"M={M}"] = {"ms_per_step": round(mq_ms, 4), "ms_per_query_token": round(mq_ms / M, 4),
                        "gb_per_s": round(step_bytes / (mq_ms * 1e-3) / 1e9, 1)}
        del q_m, out_m, ws_m

    # ---- full-depth line: the same batch in the depth-7 format (one radius per vector, 2 bits for each
    # angle of levels 5-7: 50 bytes per vector instead of 62), two rotating caches; encode and attention
    ctx_d = Context(seed=0)
    ctx_d.set_recursion_depth(7, [2, 2, 2])
    deep_caches = []
    for c in range(2):
        dkc, dkr = ctx_d.alloc_cache_for(HKV, pool, dev)
        dvc, dvr = ctx_d.alloc_cache_for(HKV, pool, dev)
        for t in (dkc, dkr, dvc, dvr):
            t.zero_()
        for b in range(B):
            k = synth.kv_stream(CTX, HKV, seed=1000 * c + 2 * b, device=dev)
            v = synth.kv_stream(CTX, HKV, seed=1000 * c + 2 * b + 1, device=dev)
            ctx_d.encode_kv(k, PQ_KEY, dkc, dkr, dst_token0=b * pool_per_seq, ld_token=k.stride(1), ld_head=k.stride(0),
                            n_tokens=CTX, n_heads=HKV)
            ctx_d.encode_kv(v, PQ_VALUE, dvc, dvr, dst_token0=b * pool_per_seq, ld_token=v.stride(1), ld_head=v.stride(0),
                            n_tokens=CTX, n_heads=HKV)
            del k, v
        deep_caches.append((dkc, dkr, dvc, dvr))

    def deep_step(i):
        kc_, kr_, vc_, vr_ = deep_caches[i % 2]
        ctx_d.decode_step_polar(new_k, new_v, newest_slot, q, out, kc_, kr_, vc_, vr_, seq_start, ctx_len, CTX, scale, ws)

    for i in range(args.warmup):
        deep_step(i)
    torch.cuda.synchronize()
    profile_begin(args.steps + 1, every=4)
    t0 = time.perf_counter()
    for i in range(args.steps):
        deep_step(i)
    torch.cuda.synchronize()
    deep_ms = 1e3 * (time.perf_counter() - t0) / args.steps
    pr_d = profile_end()
    deep_kern_ms = pr_d["attn_ms"] / max(pr_d["attn_launches"], 1)
    deep_bytes = 2 * 50 * B * HKV * CTX

    def encode_step_d(i):
        k, v, slot0 = enc_inputs[i % len(enc_inputs)]
        dkc, dkr, dvc, dvr = deep_caches[0]
        ctx_d.encode_kv_pair(k, v, dkc, dkr, dvc, dvr, dst_token0=slot0, ld_token=k.stride(1), ld_head=k.stride(0),
                             n_tokens=CTX, n_heads=HKV)

    for i in range(args.warmup):
        encode_step_d(i)
    torch.cuda.synchronize()
    profile_begin(2 * args.encode_steps + 2)
    for i in range(args.encode_steps):
        encode_step_d(i)
    torch.cuda.synchronize()
    pr_de = profile_end()
    enc_d_mtok = CTX * args.encode_steps / (pr_de["encode_ms"] * 1e-3) / 1e6 if pr_de["encode_ms"] > 0 else 0.0
    del deep_caches

    cache0 = caches[0]  # kept for the CPU baseline's cross-check
    del caches, enc_inputs, win_k, win_v, ws_h
    torch.cuda.empty_cache()

    # ---- long-context line (configs[3]): batch 4, 131072-token context; decode step on two rotating caches
    # and the bulk encoder over the full context (4 sequences x 8 heads x 131072 tokens, keys and values)
    B3, CTX3 = 4, 131072
    pool3_per_seq = CTX3 + 64
    seq_start3 = torch.arange(B3, dtype=torch.int64, device=dev) * pool3_per_seq
    ctx_len3 = torch.full((B3,), CTX3, dtype=torch.int32, device=dev)
    newest3 = seq_start3 + (CTX3 - 1)
    caches3, enc3_inputs = [], []
    for c in range(2):
        kc, kr = Context.alloc_cache(HKV, B3 * pool3_per_seq, dev)
        vc, vr = Context.alloc_cache(HKV, B3 * pool3_per_seq, dev)
        for t in (kc, kr, vc, vr):
            t.zero_()
        for b in range(B3):
            k = synth.kv_stream(CTX3, HKV, seed=3000 + 100 * c + 2 * b, device=dev)
            v = synth.kv_stream(CTX3, HKV, seed=3000 + 100 * c + 2 * b + 1, device=dev)
            ctx.encode_kv_pair(k, v, kc, kr, vc, vr, dst_token0=b * pool3_per_seq, ld_token=k.stride(1),
                               ld_head=k.stride(0), n_tokens=CTX3, n_heads=HKV)
            if c == 0:
                enc3_inputs.append((k, v, b * pool3_per_seq))
            del k, v
        caches3.append((kc, kr, vc, vr))
    ws3 = torch.empty(Context.attn_workspace_bytes(B3, HQ, HKV, CTX3), dtype=torch.uint8, device=dev)
    q3, out3 = q[:B3].contiguous(), torch.empty((B3, HQ, D), dtype=torch.bfloat16, device=dev)
    new_k3, new_v3 = new_k[:B3].contiguous(), new_v[:B3].contiguous()

    def long_step(i):
        kc_, kr_, vc_, vr_ = caches3[i % 2]
        ctx.decode_step_polar(new_k3, new_v3, newest3, q3, out3, kc_, kr_, vc_, vr_, seq_start3, ctx_len3, CTX3, scale, ws3)

    for i in range(args.warmup):
        long_step(i)
    torch.cuda.synchronize()
    profile_begin(args.steps + 1, every=4)
    t0 = time.perf_counter()
    for i in range(args.steps):
        long_step(i)
    torch.cuda.synchronize()
    long_ms = 1e3 * (time.perf_counter() - t0) / args.steps
    pr_l = profile_end()
    long_kern_ms = pr_l["attn_ms"] / max(pr_l["attn_launches"], 1)
    long_bytes = BYTES_PER_TOKEN_HEAD * B3 * HKV * CTX3

    def encode_step3(i):
        k, v, slot0 = enc3_inputs[i % B3]
        kc_, kr_, vc_, vr_ = caches3[0]
        ctx.encode_kv_pair(k, v, kc_, kr_, vc_, vr_, dst_token0=slot0, ld_token=k.stride(1), ld_head=k.stride(0),
                           n_tokens=CTX3, n_heads=HKV)

    for i in range(B3):
        encode_step3(i)
    torch.cuda.synchronize()
    enc3_launches = 3 * B3  # the full context of the batch, three times over
    profile_begin(2 * enc3_launches + 2)
    for i in range(enc3_launches):
        encode_step3(i)
    torch.cuda.synchronize()
    pr_e3 = profile_end()
    enc3_mtok = CTX3 * enc3_launches / (pr_e3["encode_ms"] * 1e-3) / 1e6 if pr_e3["encode_ms"] > 0 else 0.0
    del caches3, enc3_inputs, ws3
    torch.cuda.empty_cache()

    # ---- ragged serving line (configs[4]): 64 sequences with context lengths uniform in [1024, 65536]; one
    # step = 32 layers, each with its own cache buffers: append one new token per sequence, then attend
    B4, LAYERS = 64, 32
    lens4 = [int(n) for n in synth.ragged_lengths(B4, 1024, 65536, seed=4)]
    starts4, pos = [], 0
    for n in lens4:
        starts4.append(pos)
        pos += ((n + 63) // 64) * 64 + 64
    pool4 = pos
    seq_start4 = torch.tensor(starts4, dtype=torch.int64, device=dev)
    ctx_len4 = torch.tensor(lens4, dtype=torch.int32, device=dev)
    newest4 = seq_start4 + ctx_len4.to(torch.int64) - 1
    kc, kr = Context.alloc_cache(HKV, pool4, dev)
    vc, vr = Context.alloc_cache(HKV, pool4, dev)
    for t in (kc, kr, vc, vr):
        t.zero_()
    for b, n in enumerate(lens4):
        k = synth.kv_stream(n, HKV, seed=4000 + 2 * b, device=dev)
        v = synth.kv_stream(n, HKV, seed=4000 + 2 * b + 1, device=dev)
        ctx.encode_kv_pair(k, v, kc, kr, vc, vr, dst_token0=starts4[b], ld_token=k.stride(1), ld_head=k.stride(0),
                           n_tokens=n, n_heads=HKV)
        del k, v
    layers4 = [(kc, kr, vc, vr)] + [tuple(t.clone() for t in (kc, kr, vc, vr)) for _ in range(LAYERS - 1)]
    max_ctx4 = max(lens4)
    ws4 = torch.empty(Context.attn_workspace_bytes(B4, HQ, HKV, max_ctx4), dtype=torch.uint8, device=dev)
    q4 = synth.queries(B4, HQ, seed=14, device=dev)
    out4 = torch.empty((B4, HQ, D), dtype=torch.bfloat16, device=dev)
    new_k4 = synth.kv_stream(B4, HKV, seed=15, device=dev).permute(1, 0, 2).contiguous()
    new_v4 = synth.kv_stream(B4, HKV, seed=16, device=dev).permute(1, 0, 2).contiguous()

    def ragged_step():
        for kc_, kr_, vc_, vr_ in layers4:
            ctx.decode_step_polar(new_k4, new_v4, newest4, q4, out4, kc_, kr_, vc_, vr_, seq_start4, ctx_len4,
                                  max_ctx4, scale, ws4)

    ragged_steps = max(args.steps // 20, 2)
    ragged_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(ragged_steps):
        ragged_step()
    torch.cuda.synchronize()
    ragged_ms = 1e3 * (time.perf_counter() - t0) / ragged_steps
    ragged_bytes = BYTES_PER_TOKEN_HEAD * HKV * sum(lens4) * LAYERS
    del layers4, kc, kr, vc, vr, ws4
    torch.cuda.empty_cache()

    # ---- counter figures of the dominant kernel (separate profiling runs of this script, kept in profiles/) ----
    figures = profile_figures()
    traffic = None
    if "fetch_bytes_per_launch" in figures and "write_bytes_per_launch" in figures:
        traffic = float(figures["fetch_bytes_per_launch"]) + float(figures["write_bytes_per_launch"])
    roofline_alu = None
    if "sq_insts_valu_per_launch" in figures and kern_ms > 0:
        valu = float(figures["sq_insts_valu_per_launch"])  # executed wavefront vector instructions, matrix ones included
        ginstr = valu / (kern_ms * 1e-3) / 1e9
        roofline_alu = {
            "bound": "alu",
            "kernel": "pq_attn_partial_kernel",
            "achieved": round(ginstr, 1),
            "peak": VALU_PEAK_GINSTR,
            "unit": "G wavefront vector instructions/s",
            "frac": round(ginstr / VALU_PEAK_GINSTR, 4),
            "instructions_per_launch": valu,
            "note": "count-based: the peak is one wavefront instruction per SIMD every 4 cycles (integer three-operand and "
                    "packed binary16 instructions; fp32 and shifts take 2, matrix instructions 8 or 16)",
            "source": "SQ_INSTS_VALU of a separate rocprofv3 run (" + os.path.relpath(PROFILE_FILE, ROOT) + ", commit "
                      + figures.get("commit", "?") + ") over the launch duration measured here",
        }

    result = {
        "metric": "decode attn HBM GB/s on polar-quantized KV @32k ctx",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {
            "workload": "configs[2]: GQA decode attention, batch 16, 32 q heads / 8 kv heads, 32768-token context, d=128; "
                        "step = pq_decode_step_polar: append newest K and V token per sequence, then attention on the packed cache",
            "batch": B, "q_heads": HQ, "kv_heads": HKV, "context": CTX, "rotating_caches": N_CACHES,
            "algorithmic_bytes_per_step": step_bytes,
        },
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "roofline": {
            "bound": "hbm",
            "kernel": "pq_attn_partial_kernel",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated; separate profiling runs, "
                            "figures from " + os.path.relpath(PROFILE_FILE, ROOT) + ", taken on commit " + figures.get("commit", "?") + ")",
            "kernel_avg_ms": round(kern_ms, 5),
            "launches_timed": prof["attn_launches"],
        },
        "roofline_alu": roofline_alu,
        "encode": {
            "workload": "configs[1]: 8 kv heads x 32768 tokens, bf16 keys and values with outlier channels",
            "mtok_per_s": round(enc_mtok, 2),
            "gb_per_s": round(enc_gbs, 1),
            "frac_of_hbm_roofline": round(enc_gbs / HBM_PEAK_GBS, 4),
            "kernel": "pq_encode_kernel",
            "tokens_timed": encode_tokens,
        },
        "encode_hadamard": {
            "workload": "configs[1] with S = randomised Hadamard matrix (pq_init_preconditioner_hadamard)",
            "mtok_per_s": round(enc_h_mtok, 2),
            "gb_per_s": round(enc_h_mtok * 1e6 * enc_bytes_per_token / 1e9, 1),
            "frac_of_hbm_roofline": round(enc_h_mtok * 1e6 * enc_bytes_per_token / 1e9 / HBM_PEAK_GBS, 4),
        },
        "fit": {
            "workload": "online codebooks (Section 4.1) from the keys of one configs[1] sequence: pq_fit_count_angles "
                        "(clear, rotate, polar transform, 120 angles per vector into histograms) on the launch stream, "
                        "then pq_fit_cluster (10 k-means rounds on the counts, host)",
            "vectors": fit_vectors,
            "count_ms": round(fit_ms, 4),
            "g_vectors_per_s": round(fit_vectors / (fit_ms * 1e-3) / 1e9, 3),
            "frac_of_hbm_roofline": round(fit_vectors * 256 / (fit_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),  # 256 B read per vector
            "cluster_rounds": 10,
            "cluster_host_ms": round(fit_host_ms, 3),
        },
        "general_format": {
            "workload": "the plain path for other bit widths and recursion depths (pq_general_*), depth 5, bits 4/2/2/2/2 "
                        "(55 bytes per vector): encode of 65536 bf16 vectors; attention of 4 sequences x 2048 tokens, "
                        "8 q / 2 kv heads; generic bit reader, fp32, one wavefront per vector, sixteen per (sequence, head): not tuned",
            "encode_ms": round(g_enc_ms, 4),
            "encode_m_vectors_per_s": round(g_n / (g_enc_ms * 1e-3) / 1e6, 1),
            "attention_ms": round(g_attn_ms, 4),
            "attention_m_tokens_per_s": round(g_B * g_hq * g_ctx / (g_attn_ms * 1e-3) / 1e6, 2),
        },
        "hybrid": {
            "workload": "configs[2] prefix + 256 unquantised (bf16) recent tokens per sequence, pq_attn_decode_hybrid "
                        "(attention only, no append)",
            "ms_per_step": round(hybrid_ms, 4),
            "gb_per_s": round(hybrid_bytes / (hybrid_ms * 1e-3) / 1e9, 1),
            "algorithmic_bytes_per_step": hybrid_bytes,
        },
        "multi_query": {
            "workload": "configs[2] cache, M query tokens per sequence under the causal mask, pq_attn_decode_polar_mq "
                        "(attention only); gb_per_s counts the packed cache once per step",
            **mq,
        },
        "full_depth": {
            "workload": "configs[2] in the depth-7 format (pq_set_recursion_depth(7, {2,2,2}): 50 bytes per vector), "
                        "pq_decode_step_polar; encode: configs[1] inputs",
            "ms_per_step": round(deep_ms, 4),
            "kernel_avg_ms": round(deep_kern_ms, 5),
            "gb_per_s": round(deep_bytes / (deep_ms * 1e-3) / 1e9, 1),
            "algorithmic_bytes_per_step": deep_bytes,
            "encode_mtok_per_s": round(enc_d_mtok, 2),
        },
        "long_context": {
            "workload": "configs[3]: batch 4, 32 q heads / 8 kv heads, 131072-token context, decode step on two rotating "
                        "caches; encode = pq_encode_kv_pair over the full context (8.39 M vectors)",
            "ms_per_step": round(long_ms, 4),
            "kernel_avg_ms": round(long_kern_ms, 5),
            "gb_per_s": round(long_bytes / (long_ms * 1e-3) / 1e9, 1),
            "pct_of_hbm_peak": round(100.0 * long_bytes / (long_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
            "algorithmic_bytes_per_step": long_bytes,
            "encode_mtok_per_s": round(enc3_mtok, 2),
        },
        "ragged_serving": {
            "workload": "configs[4]: 64 sequences, context lengths uniform in [1024, 65536] (seed 4), one step = 32 layers "
                        "with distinct cache buffers, each pq_decode_step_polar (append one token per sequence, attend)",
            "ms_per_step": round(ragged_ms, 3),
            "ms_per_layer": round(ragged_ms / LAYERS, 4),
            "gb_per_s": round(ragged_bytes / (ragged_ms * 1e-3) / 1e9, 1),
            "pct_of_hbm_peak": round(100.0 * ragged_bytes / (ragged_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
            "algorithmic_bytes_per_step": ragged_bytes,
            "tokens_in_context": sum(lens4),
            "steps_timed": ragged_steps,
        },
        "setup_s": round(t_setup, 1),
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, kept, q, scale, cache0, seq_start, ctx_len, ctx, pool_per_seq)

    print(json.dumps(result))


def cpu_baseline(args, kept, q, scale, cache0, seq_start, ctx_len, ctx, pool_per_seq):
    """The fp64 oracle, untuned, on the host cores: the same step on the first sequences of cache 0."""
    import torch

    import oracle

    n = args.cpu_sample_seqs
    S = oracle.preconditioner(0)
    cb = oracle.default_codebooks()
    k_rec = np.zeros((HKV, n * CTX, 62), dtype=np.uint8)
    v_rec = np.zeros((HKV, n * CTX, 62), dtype=np.uint8)
    t_enc = time.perf_counter()
    for b in range(n):
        k, v = kept[b]
        k_rec[:, b * CTX:(b + 1) * CTX] = oracle.encode(k.double().numpy().reshape(-1, D), S, cb).reshape(HKV, CTX, 62)
        v_rec[:, b * CTX:(b + 1) * CTX] = oracle.encode(v.double().numpy().reshape(-1, D), S, cb).reshape(HKV, CTX, 62)
    t_enc = time.perf_counter() - t_enc
    qs = q[:n].double().cpu().numpy()
    starts = np.arange(n, dtype=np.int64) * CTX
    lens = np.full(n, CTX, dtype=np.int32)
    t0 = time.perf_counter()
    ref = oracle.attention(qs, k_rec, v_rec, starts, lens, S, cb, scale)
    dt = time.perf_counter() - t0
    gbs = BYTES_PER_TOKEN_HEAD * n * HKV * CTX / dt / 1e9
    # the GPU result for the same sequences (cache 0 before any append), as a parity read-out
    kc, kr, vc, vr = cache0
    out32 = torch.empty((B, HQ, D), dtype=torch.float32, device=q.device)
    ws = torch.empty(type(ctx).attn_workspace_bytes(B, HQ, HKV, CTX), dtype=torch.uint8, device=q.device)
    # slot CTX-1 was overwritten by the timed appends; re-encode is not needed for a read-out of the
    # first CTX-1 tokens: compare on a context of CTX-1 tokens instead
    lens_gpu = ctx_len.clone()
    lens_gpu[:] = CTX - 1
    ctx.attn_decode_polar(q, out32, kc, kr, vc, vr, seq_start, lens_gpu, CTX, scale, ws)
    torch.cuda.synchronize()
    ref2 = oracle.attention(qs, k_rec, v_rec, starts, lens - 1, S, cb, scale, rotated=True)
    got = out32[:n].cpu().numpy().astype(np.float64)
    err = float(np.linalg.norm(got - ref2) / np.linalg.norm(ref2))
    return {
        "value": round(gbs, 5),
        "unit": "GB/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"attention of the first {n} of 16 sequences (all 8 kv heads, 32768 tokens each), fp64, "
                  f"{dt:.1f} s; its cache was encoded by the oracle in {t_enc:.1f} s "
                  f"({2 * n * HKV * CTX / t_enc / 1e3:.0f} k vectors/s, not part of the timed figure)",
        "seconds": round(dt, 2),
        "gpu_vs_oracle_rel_l2_on_sample": round(err, 6),
    }


if __name__ == "__main__":
    main()
