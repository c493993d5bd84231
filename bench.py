"""Benchmark of the TaDA KV-cache hot path on one MI355X.

Workload (the full-cache configuration of the baseline): Llama-3-8B shape, 32 layers, 32 query /
8 kv heads, head_dim 128, batch 16, context 32768, bf16, group size 32, per-layer bit map seeded
from {2,4,8} with about a quarter of the layers at 8 bits, per-channel block mean.  The cache is
filled by bulk quantise-append (untimed warm-up of the state, reported separately), then one
"step" = for every layer: append one new token per sequence, then decode attention over the whole
cache.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is the decode-attention algorithmic bytes of the timed steps divided
by the wall time of those steps (appends included), in GB/s.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published
# HBM bytes per launch of the decode split kernel divided by its algorithmic bytes, from the
# FETCH_SIZE / WRITE_SIZE counter runs summarised in profiles/hot_path_kernels_hbm_traffic.txt
# (counters scaled by what they read for a plain copy of known size: x2.000 and x1.000)
TRAFFIC_RATIO = {2: 1.005, 4: 1.002, 8: 1.000}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--context", type=int, default=32768)
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--path", type=int, default=0, help="0 auto, 1 vector-ALU kernels, 2 matrix-core kernels")
    ap.add_argument("--q-heads", type=int, default=32)
    ap.add_argument("--kv-heads", type=int, default=8)
    ap.add_argument("--group", type=int, default=32, help="group size G = Gc")
    ap.add_argument("--paged", action="store_true", help="paged placement: block slots in a shuffled order through a block table")
    ap.add_argument("--resid", type=int, default=0, help="raw-token buffer length R, a multiple of G (0: R = G; the paper uses 128)")
    ap.add_argument("--scheme", default="mixed248", help="layer bit map: mixed248 or mixed24_8ends")
    ap.add_argument("--seed", type=int, default=2000)
    ap.add_argument("--splits", type=int, default=0, help="force the sequence split count (0 = automatic)")
    ap.add_argument("--mean-mode", default="channel", choices=["channel", "cross", "none"],
                    help="channel: per-channel block mean (the workload); cross: mean over kv heads (Eq. 1-2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-append", dest="fused_step", action="store_false",
                    help="append and attend as two calls per layer instead of the one-call decode step")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2506_04642_amd import binding as kv
    from paper_2506_04642_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    L, B, Hq, Hkv, d, G = args.layers, args.batch, args.q_heads, args.kv_heads, 128, args.group
    T0 = args.context
    K, W = args.steps, args.warmup
    n_dec = K + W
    max_tokens = (T0 + n_dec + 8 + G - 1) // G * G
    bits = synth.layer_bits(args.seed, L, args.scheme)
    mean_mode = {"channel": kv.KV_MEAN_CHANNEL_BLOCK, "cross": kv.KV_MEAN_CROSS_HEAD, "none": kv.KV_MEAN_NONE}[args.mean_mode]
    R = args.resid if args.resid else G  # raw trailing tokens are compressed R at a time (Sec. 3.3)
    max_tokens = (max_tokens + R - 1) // R * R
    pool = B * (max_tokens // G) if args.paged else 0
    cfg = kv.make_config(L, B, Hq, Hkv, d, max_tokens, G, G, R, kv.KV_BF16, mean_mode, bits, bits, pool_blocks=pool)
    cache = kv.KVCache(cfg, device=dev, zero=False)
    if args.paged:
        perm = np.random.default_rng(args.seed).permutation(pool).astype(np.int32).reshape(B, max_tokens // G)
        cache.set_block_table(torch.from_numpy(perm).to(dev))
    kv.kv_set_decode_path(cache.handle, args.path)
    if args.splits:
        kv.kv_set_decode_splits(cache.handle, args.splits)
        cache.ws_bytes = max(cache.ws_bytes, B * Hq * args.splits * 132 * 4)
        cache.workspace = torch.empty(cache.ws_bytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev)

    # ---- fill: bulk quantise-append in chunks, inputs drawn on the device
    sample_layers = {}
    for b_ in (2, 4, 8):
        if b_ in bits:
            sample_layers[bits.index(b_)] = b_
    host_kv = {}
    NS = min(4, B)  # sequences of the batch that the CPU oracle re-does (about 10 s of one core)
    chunk = 4096
    fill_ms = 0.0
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for l in range(L):
        keep = l in sample_layers and not args.no_cpu_baseline
        hk, hv = [], []
        for t0 in range(0, T0, chunk):
            n = min(chunk, T0 - t0)
            k, v = synth.make_kv_torch(2000 * 1000 + l * 64 + t0 // chunk, B, n, Hkv, d, synth.BF16, dev)
            ev0.record(stream)
            cache.append(l, k, v)
            ev1.record(stream)
            ev1.synchronize()
            fill_ms += ev0.elapsed_time(ev1)
            if keep:
                hk.append(k[0:NS].cpu())
                hv.append(v[0:NS].cpu())
            del k, v
        if keep:
            host_kv[l] = (torch.cat(hk, 1), torch.cat(hv, 1))
    bulk_tokens = L * B * T0

    # ---- decode inputs (resident before timing)
    k_dec = [synth.make_kv_torch(77000 + l, B, n_dec, Hkv, d, synth.BF16, dev) for l in range(L)]
    q_dec = [synth.make_q_torch(88000 + l, B, Hq, d, synth.BF16, dev) for l in range(L)]
    out = torch.empty((B, Hq, d), dtype=torch.float32, device=dev)
    ws, wsb = cache.workspace.data_ptr(), cache.ws_bytes
    sp = stream.cuda_stream

    def step(s, events=None):
        nbytes = 0
        for l in range(L):
            kd, vd = k_dec[l]
            fused = args.fused_step and cache.lengths(l)[1] + 1 < R  # the token does not fill the raw buffer
            if not fused:
                cache.append(l, kd[:, s:s + 1], vd[:, s:s + 1])
            if events is not None:
                e0, e1 = events[l]
                e0.record(stream)
            if fused:
                # the attention kernel takes the new token from the caller's rows and stores it
                kn, vn = kd[:, s], vd[:, s]
                kv.kv_append_decode_attn_split(cache.handle, l, kn.data_ptr(), vn.data_ptr(), kn.stride(0),
                                               kn.stride(1), q_dec[l].data_ptr(), ws, wsb, sp)
            else:
                kv.kv_decode_attn_split(cache.handle, l, q_dec[l].data_ptr(), ws, wsb, sp)
            if events is not None:
                e1.record(stream)
            kv.kv_decode_attn_merge(cache.handle, l, out.data_ptr(), ws, wsb, sp)
            nbytes += kv.kv_decode_bytes(cache.handle, l)
        return nbytes

    for s in range(W):
        step(s)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps, HIP events around every split kernel on the launch stream
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(L)]
           for _ in range(K)]
    layer_bytes = [0] * L
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    total_bytes = 0
    for s in range(K):
        total_bytes += step(W + s, evs[s])
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    wall = t_end - t_start
    for l in range(L):
        layer_bytes[l] = kv.kv_decode_bytes(cache.handle, l)

    split_ms = np.array([[evs[s][l][0].elapsed_time(evs[s][l][1]) for l in range(L)] for s in range(K)])
    per_bits = {}
    # the counter runs were made on the matrix-core kernels of the default format
    traffic_known = args.path != 1 and args.group == 32 and args.mean_mode == "channel" and not args.paged
    for b_ in sorted(set(bits)):
        idx = [l for l in range(L) if bits[l] == b_]
        ms = float(split_ms[:, idx].mean())
        byts = float(np.mean([layer_bytes[l] for l in idx]))
        per_bits[str(b_)] = {"layers": len(idx), "splits": kv.kv_decode_splits(cache.handle, idx[0]),
                             "avg_ms": round(ms, 5), "median_ms": round(float(np.median(split_ms[:, idx])), 5),
                             "p10_ms": round(float(np.percentile(split_ms[:, idx], 10)), 5),
                             "p90_ms": round(float(np.percentile(split_ms[:, idx], 90)), 5), "bytes": int(byts),
                             "GBps": round(byts / ms / 1e6, 1), "frac": round(byts / ms / 1e6 / HBM_PEAK_GBPS, 4),
                             "traffic": int(byts * TRAFFIC_RATIO[b_]) if b_ in TRAFFIC_RATIO and traffic_known else None}
    achieved = float(sum(layer_bytes)) / float(split_ms.mean(axis=0).sum()) / 1e6
    traffic = None
    if traffic_known and all(b_ in TRAFFIC_RATIO for b_ in bits):
        traffic = int(sum(layer_bytes[l] * TRAFFIC_RATIO[bits[l]] for l in range(L)) / L)

    # ---- what a plain streaming read of the same size reaches on this machine (context for `frac`):
    # torch's int64 sum over a buffer as large as one layer's algorithmic bytes, rotated over a pool
    ceiling = {}
    pool = torch.ones(2 * 1024 ** 3 // 8, dtype=torch.int64, device=dev)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for b_ in sorted(set(bits)):
        n = min(per_bits[str(b_)]["bytes"] // 8, pool.numel())
        views = [pool[i * n:(i + 1) * n] for i in range(max(1, pool.numel() // n))]
        for v_ in views[:2]:
            v_.sum()
        ts = []
        for it in range(12):
            c0.record(stream)
            views[it % len(views)].sum()
            c1.record(stream)
            c1.synchronize()
            ts.append(c0.elapsed_time(c1))
        ts.sort()
        ceiling[str(b_)] = round(n * 8 / ts[len(ts) // 2] / 1e6, 1)
        per_bits[str(b_)]["frac_of_stream_read"] = round(per_bits[str(b_)]["GBps"] / ceiling[str(b_)], 4)
    del pool

    # ---- context only: one layer of the same shape as a 16-bit cache, attended by torch's own
    # scaled_dot_product_attention (not tuned for decode) -- what the packed cache is an alternative to
    sdpa_ctx = None
    try:
        import torch.nn.functional as F

        kb = torch.randn((B, Hkv, T0, d), device=dev, dtype=torch.bfloat16)
        vb = torch.randn((B, Hkv, T0, d), device=dev, dtype=torch.bfloat16)
        qb = torch.randn((B, Hkv, Hq // Hkv, d), device=dev, dtype=torch.bfloat16)
        for _ in range(2):
            F.scaled_dot_product_attention(qb, kb, vb)
        ts = []
        for _ in range(8):
            c0.record(stream)
            F.scaled_dot_product_attention(qb, kb, vb)
            c1.record(stream)
            c1.synchronize()
            ts.append(c0.elapsed_time(c1))
        ts.sort()
        raw_bytes = 2 * B * Hkv * T0 * d * 2
        sdpa_ctx = {"bytes_per_layer": raw_bytes, "torch_sdpa_ms_per_layer": round(ts[len(ts) // 2], 4),
                    "ms_at_hbm_peak": round(raw_bytes / HBM_PEAK_GBPS / 1e6, 4)}
        del kb, vb, qb
    except Exception as ex:  # context only: the line is valid without it
        sdpa_ctx = {"error": repr(ex)[:120]}

    # ---- single-token append cost, measured apart from the timed region
    torch.cuda.synchronize()
    app_t0 = time.perf_counter()
    # (host-side only bookkeeping would be skipped by a no-op; use the real call on spare capacity)
    spare = max_tokens - (T0 + n_dec)
    n_app = min(spare, 8)
    for s in range(n_app):
        for l in range(L):
            kd, vd = k_dec[l]
            cache.append(l, kd[:, s:s + 1], vd[:, s:s + 1])
    torch.cuda.synchronize()
    app_s = time.perf_counter() - app_t0

    # ---- rotation fused into the bulk append (Alg. 1 step 5), on a scratch cache of one layer per
    # bit width: the same 4096-token chunks through kv_quant_append and through kv_rope_quant_append
    rope_stats = {}
    n_rope = 4096
    sbits = sorted(set(bits))
    scfg = kv.make_config(len(sbits), B, Hq, Hkv, d, 2 * n_rope, G, G, G, kv.KV_BF16, kv.KV_MEAN_CHANNEL_BLOCK, sbits, sbits)
    scratch = kv.KVCache(scfg, device=dev, zero=False)
    kr, vr = synth.make_kv_torch(4242, B, n_rope, Hkv, d, synth.BF16, dev)
    cos_h, sin_h = synth.rope_tables(np.arange(n_rope), d)
    cos_d, sin_d = torch.from_numpy(cos_h).to(dev), torch.from_numpy(sin_h).to(dev)
    for fused in (False, True):
        ts = []
        for rep in range(4):
            kv.kv_cache_reset(scratch.handle, -1)
            torch.cuda.synchronize()
            c0.record(stream)
            for l in range(len(sbits)):
                if fused:
                    scratch.append_rope(l, kr, vr, cos_d, sin_d, kv.KV_ROPE_HALF)
                else:
                    scratch.append(l, kr, vr)
            c1.record(stream)
            c1.synchronize()
            ts.append(c0.elapsed_time(c1))
        ms = sorted(ts[1:])[len(ts[1:]) // 2]
        tok = len(sbits) * B * n_rope
        rope_stats["rope_fused" if fused else "plain"] = {
            "tokens_per_s": round(tok / (ms / 1e3), 1),
            "input_GBps": round(tok * Hkv * d * 2 * 2 / (ms / 1e3) / 1e9, 1)}
    scratch.close()
    del scratch, kr, vr

    result = {
        "metric": "decode_attn_effective_hbm_GBps",
        "value": round(total_bytes / wall / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(wall / K * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "i8 x i8 -> i32 contractions, f32 softmax" if args.path != 1 else "f32",
        "data": "synthetic",
        "config": {"workload": "llama-shaped full cache: %d layers, %dq/%dkv heads, head_dim 128, "
                               "batch %d, context %d, bf16, G=Gc=%d, %s layer bit map (seed %d), "
                               "%s" % (L, Hq, Hkv, B, T0, G, args.scheme, args.seed,
                                       {"channel": "per-channel block mean", "cross": "cross-head mean",
                                        "none": "no mean"}[args.mean_mode]),
                   "layers": L, "batch": B, "context": T0, "bit_map": bits, "decode_path": args.path},
        "pct_of_hbm_peak": round(total_bytes / wall / 1e9 / HBM_PEAK_GBPS * 100, 2),
        "decode_tokens_per_s": round(B * K / wall, 1),
        "quant_append": {
            "bulk_tokens_per_s": round(bulk_tokens / (fill_ms / 1e3), 1),
            "bulk_input_GBps": round(bulk_tokens * Hkv * d * 2 * 2 / (fill_ms / 1e3) / 1e9, 1),
            "single_token_tokens_per_s": round(B * n_app / app_s, 1) if n_app else None,
            "single_token_us_per_layer_call": round(app_s / max(n_app * L, 1) * 1e6, 2) if n_app else None,
            "bulk_4096_token_calls": rope_stats,
        },
        "roofline": {"bound": "hbm", "kernel": "decode split kernel (all layers, weighted by layer)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "bytes_per_launch": int(sum(layer_bytes) / L), "per_bits": per_bits,
                     "stream_read_GBps_same_size": ceiling},
        "context_16bit_cache": sdpa_ctx,
    }

    # ---- CPU oracle on a bounded sample of the same workload (rank 0, one core)
    if not args.no_cpu_baseline and host_kv:
        import oracle

        ocfg_bits = [sample_layers[l] for l in sorted(sample_layers)]
        nl = len(ocfg_bits)
        ocfg = oracle.OracleConfig(nl, NS, Hq, Hkv, d, max_tokens, G, G, G, oracle.tada.BF16,
                                   mean_mode, ocfg_bits, ocfg_bits)
        orc = oracle.OracleCache(ocfg)
        enc_s = att_s = 0.0
        att_bytes = 0
        worst = 0.0
        for i, l in enumerate(sorted(sample_layers)):
            hk, hv = host_kv[l]
            k16 = hk.view(torch.int16).numpy().view(np.uint16)
            v16 = hv.view(torch.int16).numpy().view(np.uint16)
            t0 = time.perf_counter()
            orc.append(i, k16, v16)
            enc_s += time.perf_counter() - t0
            # replay the decode tokens that the GPU cache has seen, so both hold the same state
            seen = W + K + n_app
            kd, vd = k_dec[l]
            order = list(range(W + K)) + list(range(n_app))
            for s in order[:seen]:
                orc.append(i, kd[0:NS, s:s + 1].cpu().view(torch.int16).numpy().view(np.uint16),
                           vd[0:NS, s:s + 1].cpu().view(torch.int16).numpy().view(np.uint16))
            q16 = q_dec[l][0:NS].cpu().view(torch.int16).numpy().view(np.uint16)
            t0 = time.perf_counter()
            want = orc.attend(i, q16)
            att_s += time.perf_counter() - t0
            got = cache.attend(l, q_dec[l])
            torch.cuda.synchronize()
            worst = max(worst, float(np.max(np.abs(got[0:NS].cpu().numpy().astype(np.float64) - want))))
            att_bytes += kv.kv_decode_bytes(cache.handle, l) * NS // B
        result["cpu_baseline"] = {
            "value": round(att_bytes / att_s / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "batch elements 0-%d (%d kv-head units, full context) of one layer per bit width %s: "
                      "decode attention %.2f s; their quantise-append %.2f s = %.0f tokens/s"
                      % (NS - 1, NS * Hkv, ocfg_bits, att_s, enc_s, nl * NS * T0 / enc_s),
            "quant_append_tokens_per_s": round(nl * NS * T0 / enc_s, 1),
            "gpu_vs_oracle_max_abs_err": worst,
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
