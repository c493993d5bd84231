"""Benchmark of the TaDA KV-cache hot path on one MI355X.

Headline workload (the full-cache configuration of the baseline): Llama-3-8B shape, 32 layers, 32 query /
8 kv heads, head_dim 128, batch 16, context 32768, bf16, group size 32, per-layer bit map seeded
from {2,4,8} with about a quarter of the layers at 8 bits, per-channel block mean.  The cache is
filled by bulk quantise-append (untimed warm-up of the state, reported separately), then one
"step" = for every layer: append one new token per sequence, then decode attention over the whole
cache.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is the decode-attention algorithmic bytes of the timed steps divided
by the wall time of those steps (appends included), in GB/s.  `other_configs` carries the same
measurement, bounded to a few seconds each, on the baseline's other configurations (latency-bound
single layers, the 80-layer batch-1 long context, prefill-then-decode at batch 64), with the mean over
the kv heads (Eq. 1-2) on the headline shape, and the value projection fused with the compression
(Alg. 1 step 3) against a library matmul followed by the plain append.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 / fp16 matrix rate, published
# Counter summary that holds, per bit width, the HBM bytes per launch of the decode split kernel
# divided by its algorithmic bytes (FETCH_SIZE + WRITE_SIZE runs), and the hash of the kernel source
# the counters were taken with; `traffic` is reported only while that source is unchanged.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "decode_split_mfma_fullcache_hbm_traffic.txt")
TRAFFIC_SOURCE = os.path.join(ROOT, "paper_2506_04642_amd", "csrc", "decode_mfma.hip")


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
    ap.add_argument("--legs", default="c0,c1,c3,c4,cross,cross128,mixed,widths,compressv,graph",
                    help="other configurations measured after the headline one (comma list, or 'none')")
    ap.add_argument("--leg-steps", type=int, default=8, help="timed decode steps of each other configuration")
    return ap.parse_args()


def traffic_ratios():
    """{bits: ratio} from the committed counter summary, or (None, reason)."""
    try:
        text = open(TRAFFIC_PROFILE).read()
        sha = hashlib.sha256(open(TRAFFIC_SOURCE, "rb").read()).hexdigest()[:16]
    except OSError as ex:
        return None, "no counter summary (%s)" % ex.__class__.__name__
    m = re.search(r"^source_sha16\s+decode_mfma\.hip\s+([0-9a-f]{16})", text, re.M)
    if not m or m.group(1) != sha:
        return None, "the decode kernel's source changed since the counter runs of %s" % os.path.basename(TRAFFIC_PROFILE)
    ratios = {int(b): float(r) for b, r in re.findall(r"^traffic_ratio\s+bits=(\d+)\s+([0-9.]+)", text, re.M)}
    return (ratios, os.path.basename(TRAFFIC_PROFILE)) if ratios else (None, "no ratios in the counter summary")


class Env:
    def __init__(self):
        import numpy as np
        import torch

        from paper_2506_04642_amd import binding as kv
        from paper_2506_04642_amd import synth

        assert torch.cuda.is_available(), "bench.py needs the GPU"
        self.np, self.torch, self.kv, self.synth = np, torch, kv, synth
        self.dev = torch.device("cuda:0")
        torch.cuda.set_device(self.dev)
        self.stream = torch.cuda.current_stream(self.dev)

    def event_pair(self):
        return self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)


def run_decode_workload(env, *, L, B, Hq, Hkv, G, T0, steps, warmup, scheme, seed, Gc=0, v_bits=None, mean_mode="channel", path=0,
                        paged=False, resid=0, splits=0, fused_step=True, sample_seqs=0, shared_inputs=False, chunk=4096):
    """Fill a cache by bulk quantise-append, then time `steps` decode steps (per layer: append one token
    per sequence, attend over the whole cache).  Returns (figures, state); state keeps the cache and the
    decode inputs alive for the legs that need them.  shared_inputs: the bulk-append chunks of one layer
    are drawn once and serve every layer (the other configurations; the headline draws each layer's own)."""
    np, torch, kv, synth, dev, stream = env.np, env.torch, env.kv, env.synth, env.dev, env.stream
    d = 128
    n_dec = steps + warmup
    R = resid if resid else G  # raw trailing tokens are compressed R at a time (Sec. 3.3)
    max_tokens = (T0 + n_dec + 8 + G - 1) // G * G
    max_tokens = (max_tokens + R - 1) // R * R
    bits = synth.layer_bits(seed, L, scheme)
    mm = {"channel": kv.KV_MEAN_CHANNEL_BLOCK, "cross": kv.KV_MEAN_CROSS_HEAD, "none": kv.KV_MEAN_NONE}[mean_mode]
    pool = B * (max_tokens // G) if paged else 0
    if v_bits is not None:  # keys and values of different widths: one pair for all layers
        bits = [v_bits[0]] * L
    cfg = kv.make_config(L, B, Hq, Hkv, d, max_tokens, G, Gc or G, R, kv.KV_BF16, mm, bits, [v_bits[1]] * L if v_bits else bits,
                         pool_blocks=pool)  # (Gc = 0: Gc = G)
    cache = kv.KVCache(cfg, device=dev, zero=False)
    if paged:
        perm = np.random.default_rng(seed).permutation(pool).astype(np.int32).reshape(B, max_tokens // G)
        cache.set_block_table(torch.from_numpy(perm).to(dev))
    kv.kv_set_decode_path(cache.handle, path)
    if splits:
        kv.kv_set_decode_splits(cache.handle, splits)
        cache.ws_bytes = max(cache.ws_bytes, B * Hq * splits * 132 * 4)
        cache.workspace = torch.empty(cache.ws_bytes, dtype=torch.uint8, device=dev)

    # ---- fill: bulk quantise-append in chunks, inputs drawn on the device
    sample_layers = {}
    if sample_seqs:
        for b_ in (2, 4, 8):
            if b_ in bits:
                sample_layers[bits.index(b_)] = b_
    host_kv = {}
    fill_ms = 0.0
    ev0, ev1 = env.event_pair()
    shared = None
    for l in range(L):
        keep = l in sample_layers
        hk, hv = [], []
        for ci, t0 in enumerate(range(0, T0, chunk)):
            n = min(chunk, T0 - t0)
            if shared_inputs:
                if shared is None or shared[0].shape[1] != n:
                    shared = synth.make_kv_torch(seed * 1000 + 17, B, n, Hkv, d, synth.BF16, dev)
                k, v = shared
            else:
                k, v = synth.make_kv_torch(seed * 1000 + l * 64 + ci, B, n, Hkv, d, synth.BF16, dev)
            ev0.record(stream)
            cache.append(l, k, v)
            ev1.record(stream)
            ev1.synchronize()
            fill_ms += ev0.elapsed_time(ev1)
            if keep:
                hk.append(k[0:sample_seqs].cpu())
                hv.append(v[0:sample_seqs].cpu())
            del k, v
        if keep:
            host_kv[l] = (torch.cat(hk, 1), torch.cat(hv, 1))
    shared = None
    bulk_tokens = L * B * T0

    # ---- decode inputs (resident before timing)
    if shared_inputs:
        kd1 = synth.make_kv_torch(77000, B, n_dec, Hkv, d, synth.BF16, dev)
        qd1 = synth.make_q_torch(88000, B, Hq, d, synth.BF16, dev)
        k_dec, q_dec = [kd1] * L, [qd1] * L
    else:
        k_dec = [synth.make_kv_torch(77000 + l, B, n_dec, Hkv, d, synth.BF16, dev) for l in range(L)]
        q_dec = [synth.make_q_torch(88000 + l, B, Hq, d, synth.BF16, dev) for l in range(L)]
    out = torch.empty((B, Hq, d), dtype=torch.float32, device=dev)
    ws, wsb = cache.workspace.data_ptr(), cache.ws_bytes
    sp = stream.cuda_stream

    # layers on the matrix-core kernels have their split kernel stamp its own events
    stamped = [kv.kv_decode_path_used(cache.handle, l) == 2 for l in range(L)]

    def step(s, events=None):
        nbytes = 0
        for l in range(L):
            kd, vd = k_dec[l]
            fused = fused_step and cache.lengths(l)[1] + 1 < R  # the token does not fill the raw buffer
            if not fused:
                cache.append(l, kd[:, s:s + 1], vd[:, s:s + 1])
            if events is not None:
                e0, e1 = events[l]
                if stamped[l]:
                    # the split kernel's dispatch stamps the two events itself: its execution time, as a kernel trace
                    # reports it (events recorded around the call also count the dispatch gaps on either side)
                    kv.kv_time_next_split(e0.cuda_event, e1.cuda_event)
                else:
                    e0.record(stream)
            if fused:
                # the attention kernel takes the new token from the caller's rows and stores it
                kn, vn = kd[:, s], vd[:, s]
                kv.kv_append_decode_attn_split(cache.handle, l, kn.data_ptr(), vn.data_ptr(), kn.stride(0),
                                               kn.stride(1), q_dec[l].data_ptr(), ws, wsb, sp)
            else:
                kv.kv_decode_attn_split(cache.handle, l, q_dec[l].data_ptr(), ws, wsb, sp)
            if events is not None and not stamped[l]:
                e1.record(stream)
            kv.kv_decode_attn_merge(cache.handle, l, out.data_ptr(), ws, wsb, sp)
            nbytes += kv.kv_decode_bytes(cache.handle, l)
        return nbytes

    for s in range(warmup):
        step(s)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps, HIP events around every split kernel on the launch stream
    evs = [[env.event_pair() for _ in range(L)] for _ in range(steps)]
    for row in evs:
        for e0, e1 in row:  # (recorded once: the handles exist before a launch is given them)
            e0.record(stream)
            e1.record(stream)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    total_bytes = 0
    for s in range(steps):
        total_bytes += step(warmup + s, evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    layer_bytes = [kv.kv_decode_bytes(cache.handle, l) for l in range(L)]

    split_ms = np.array([[evs[s][l][0].elapsed_time(evs[s][l][1]) for l in range(L)] for s in range(steps)])
    per_bits = {}
    for b_ in sorted(set(bits)):
        idx = [l for l in range(L) if bits[l] == b_]
        ms = float(split_ms[:, idx].mean())
        byts = float(np.mean([layer_bytes[l] for l in idx]))
        per_bits[str(b_)] = {"layers": len(idx), "splits": kv.kv_decode_splits(cache.handle, idx[0]),
                             "avg_ms": round(ms, 5), "median_ms": round(float(np.median(split_ms[:, idx])), 5),
                             "p10_ms": round(float(np.percentile(split_ms[:, idx], 10)), 5),
                             "p90_ms": round(float(np.percentile(split_ms[:, idx], 90)), 5), "bytes": int(byts),
                             "GBps": round(byts / ms / 1e6, 1), "frac": round(byts / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    achieved = float(sum(layer_bytes)) / float(split_ms.mean(axis=0).sum()) / 1e6
    fig = {
        "value_GBps": round(total_bytes / wall / 1e9, 2), "ms_per_step": round(wall / steps * 1e3, 4),
        "pct_of_hbm_peak": round(total_bytes / wall / 1e9 / HBM_PEAK_GBPS * 100, 2),
        "decode_tokens_per_s": round(B * steps / wall, 1), "bit_map": bits,
        "split_kernels_GBps": round(achieved, 1), "split_kernels_frac_of_peak": round(achieved / HBM_PEAK_GBPS, 4),
        "bytes_per_launch": int(sum(layer_bytes) / L), "per_bits": per_bits,
        "bulk_append_tokens_per_s": round(bulk_tokens / (fill_ms / 1e3), 1),
        "bulk_append_input_GBps": round(bulk_tokens * Hkv * d * 2 * 2 / (fill_ms / 1e3) / 1e9, 1),
    }
    state = dict(cache=cache, k_dec=k_dec, q_dec=q_dec, bits=bits, max_tokens=max_tokens, n_dec=n_dec, R=R, mm=mm,
                 host_kv=host_kv, sample_layers=sample_layers, layer_bytes=layer_bytes, total_bytes=total_bytes, wall=wall)
    return fig, state


def release(env, state):
    state["cache"].close()
    state.clear()
    env.torch.cuda.empty_cache()


def stream_read_ceiling(env, sizes):
    """What the library's read-only streaming kernel reaches on buffers of the given sizes (median of 12
    passes rotated over a 2 GiB pool): the measured ceiling next to the published peak."""
    torch, kv, dev, stream = env.torch, env.kv, env.dev, env.stream
    pool = torch.ones(2 * 1024 ** 3 // 8, dtype=torch.int64, device=dev)
    c0, c1 = env.event_pair()
    res = {}
    for key, nbytes in sizes.items():
        n = min(nbytes // 16 * 16, pool.numel() * 8)
        views = max(1, pool.numel() * 8 // n)
        ts = []
        for it in range(14):
            off = (it % views) * n
            c0.record(stream)
            kv.kv_stream_read_probe(pool.data_ptr() + off, n, 0, stream.cuda_stream)
            c1.record(stream)
            c1.synchronize()
            ts.append(c0.elapsed_time(c1))
        ts = sorted(ts[2:])
        res[key] = round(n / ts[len(ts) // 2] / 1e6, 1)
    del pool
    return res


def latency_leg(env, name, *, Hq, Hkv, T, dtype_name, reps=60):
    """Single-layer configurations whose cache fits the on-chip caches: time per call, not a bandwidth."""
    np, torch, kv, synth, dev, stream = env.np, env.torch, env.kv, env.synth, env.dev, env.stream
    dt = synth.F16 if dtype_name == "fp16" else synth.BF16
    kdt = kv.KV_F16 if dtype_name == "fp16" else kv.KV_BF16
    G = 32
    cfg = kv.make_config(1, 1, Hq, Hkv, 128, (T + 64) // G * G, G, G, G, kdt, kv.KV_MEAN_CHANNEL_BLOCK, [4], [4])
    cache = kv.KVCache(cfg, device=dev, zero=False)
    k, v = synth.make_kv_torch(5, 1, T + 32, Hkv, 128, dt, dev)
    q = synth.make_q_torch(5, 1, Hq, 128, dt, dev)
    c0, c1 = env.event_pair()
    c0.record(stream)
    cache.append(0, k[:, :T - 1], v[:, :T - 1])
    c1.record(stream)
    c1.synchronize()
    bulk_ms = c0.elapsed_time(c1)
    cache.append(0, k[:, T - 1:T], v[:, T - 1:T])
    out = torch.empty((1, Hq, 128), dtype=torch.float32, device=dev)
    for _ in range(5):
        cache.attend(0, q, out)
    ts, ss = [], []
    ws, wsb, sp = cache.workspace.data_ptr(), cache.ws_bytes, stream.cuda_stream
    for _ in range(reps):
        c0.record(stream)
        cache.attend(0, q, out)
        c1.record(stream)
        c1.synchronize()
        ts.append(c0.elapsed_time(c1))
        c0.record(stream)
        kv.kv_decode_attn_split(cache.handle, 0, q.data_ptr(), ws, wsb, sp)
        c1.record(stream)
        c1.synchronize()
        ss.append(c0.elapsed_time(c1))
    nbytes = kv.kv_decode_bytes(cache.handle, 0)
    app = []
    for i in range(16):
        c0.record(stream)
        cache.append(0, k[:, T + i:T + i + 1], v[:, T + i:T + i + 1])
        c1.record(stream)
        c1.synchronize()
        app.append(c0.elapsed_time(c1))
    med = lambda x: sorted(x)[len(x) // 2]
    res = {"workload": "%s: 1 layer, batch 1, %dq/%dkv heads, context %d, %s, 4-bit, G=Gc=32" % (name, Hq, Hkv, T, dtype_name),
           "decode_attn_us": round(med(ts) * 1e3, 2), "split_kernel_us": round(med(ss) * 1e3, 2),
           "splits": kv.kv_decode_splits(cache.handle, 0), "algorithmic_bytes": nbytes,
           "GBps_cache_resident": round(nbytes / med(ts) / 1e6, 1),
           "bulk_append_us": round(bulk_ms * 1e3, 1), "single_token_append_us": round(med(app) * 1e3, 2),
           "note": "latency-bound: the packed cache fits the on-chip caches, GB/s is not an HBM rate"}
    cache.close()
    return res


def graph_leg(env, fig, state, *, reps=4, launches=3):
    """Decode steps replayed from one HIP graph (kv_decode_step_dev: the kernels take the lengths from
    device memory and advance them) on the cache of a finished decode workload, against that
    workload's eager steps."""
    torch, kv, stream = env.torch, env.kv, env.stream
    cache, k_dec, q_dec = state["cache"], state["k_dec"], state["q_dec"]
    L = len(state["bits"])
    B, Hq, d = q_dec[0].shape
    outs = [torch.empty((B, Hq, d), dtype=torch.float32, device=env.dev) for _ in range(L)]
    ks = [k_dec[l][0][:, 0].contiguous() for l in range(L)]
    vs = [k_dec[l][1][:, 0].contiguous() for l in range(L)]

    def steps_all():
        for l in range(L):
            cache.step_dev(l, ks[l], vs[l], q_dec[l], outs[l])

    cache.lengths_to_device()
    steps_all()  # one eager step: one-time queries happen outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        steps_all()
    torch.cuda.synchronize()
    graph.replay()  # warm
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        graph.replay()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    cache.advance(reps + 2)
    nbytes = sum(kv.kv_decode_bytes(cache.handle, l) for l in range(L))
    return {"workload": "the decode steps of the leg before, every layer's step recorded once (kv_decode_step_dev: store and "
                        "quantise if the raw buffer fills, attention, merge) and replayed from one HIP graph",
            "layers": L, "launches_per_step": launches * L, "ms_per_step_graph": round(wall / reps * 1e3, 4),
            "ms_per_step_eager": fig["ms_per_step"], "value_GBps_graph": round(nbytes * reps / wall / 1e9, 2),
            "value_GBps_eager": fig["value_GBps"]}


def compressv_leg(env, *, B, n, model_dim=4096, Hkv=8, bits=4, reps=6):
    """Alg. 1 step 3: the value projection fused with the compression (kv_compressv_append) against a
    library matmul that writes the values followed by kv_quant_append, on one bulk call of B x n tokens and
    on single-token decode steps."""
    torch, kv, synth, dev, stream = env.torch, env.kv, env.synth, env.dev, env.stream
    cfg = kv.make_config(1, B, 4 * Hkv, Hkv, 128, n + 64, 32, 32, 32, kv.KV_BF16, kv.KV_MEAN_CHANNEL_BLOCK, [bits], [bits])
    c = kv.KVCache(cfg, device=dev, zero=False)
    k, _ = synth.make_kv_torch(1, B, n, Hkv, 128, synth.BF16, dev)
    x, w = synth.make_xw_torch(1, B, n, model_dim, Hkv * 128, synth.BF16, dev)
    e0, e1 = env.event_pair()

    def timeit(f):
        ts = []
        for _ in range(reps):
            kv.kv_cache_reset(c.handle, -1)
            torch.cuda.synchronize()
            e0.record(stream)
            f()
            e1.record(stream)
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        ts = sorted(ts[1:])
        return ts[len(ts) // 2]

    def separate():
        c.append(0, k, torch.matmul(x, w.t()).view(B, n, Hkv, 128))

    flops = 2.0 * B * n * model_dim * Hkv * 128
    t_f, t_s = timeit(lambda: c.append_compressv(0, k, x, w)), timeit(separate)
    t_mm, t_app = timeit(lambda: torch.matmul(x, w.t())), timeit(lambda: c.append(0, k, k))
    k1, x1 = k[:, :1].contiguous(), x[:, :1].contiguous()

    def dec_f():
        for _ in range(20):
            c.append_compressv(0, k1, x1, w)

    def dec_s():
        for _ in range(20):
            c.append(0, k1, torch.matmul(x1, w.t()).view(B, 1, Hkv, 128))

    res = {"workload": "batch %d x %d tokens per call, model_dim %d, %d kv heads, bf16, %d-bit, G=Gc=32" % (B, n, model_dim, Hkv, bits),
           "fused_ms": round(t_f, 4), "matmul_then_append_ms": round(t_s, 4), "library_matmul_ms": round(t_mm, 4),
           "plain_append_ms": round(t_app, 4), "fused_vs_separate": round(t_s / t_f, 3),
           "fused_TFLOPs": round(flops / t_f / 1e9, 1),
           "roofline": {"bound": "mfma", "achieved": round(flops / t_f / 1e9, 1), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(flops / t_f / 1e9 / MFMA_PEAK_TFLOPS, 4),
                        "note": "whole call (the keys' append launch included) against the published dense bf16 rate"},
           "decode_step_fused_us": round(timeit(dec_f) * 50, 2), "decode_step_matmul_then_append_us": round(timeit(dec_s) * 50, 2)}
    c.close()
    del k, x, w
    torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    env = Env()
    np, torch, kv, synth, dev, stream = env.np, env.torch, env.kv, env.synth, env.dev, env.stream

    L, B, Hq, Hkv, d, G = args.layers, args.batch, args.q_heads, args.kv_heads, 128, args.group
    T0, K, W = args.context, args.steps, args.warmup
    NS = 0 if args.no_cpu_baseline else min(4, B)  # sequences of the batch that the CPU oracle re-does
    fig, st = run_decode_workload(env, L=L, B=B, Hq=Hq, Hkv=Hkv, G=G, T0=T0, steps=K, warmup=W, scheme=args.scheme,
                                  seed=args.seed, mean_mode=args.mean_mode, path=args.path, paged=args.paged,
                                  resid=args.resid, splits=args.splits, fused_step=args.fused_step, sample_seqs=NS)
    cache, k_dec, q_dec, bits = st["cache"], st["k_dec"], st["q_dec"], st["bits"]
    max_tokens, n_dec, R = st["max_tokens"], st["n_dec"], st["R"]
    per_bits = fig["per_bits"]

    # ---- HBM traffic per launch from the committed counter runs, while the kernel they measured is the one built
    traffic = None
    traffic_source = None
    counters_cover = args.path != 1 and args.group == 32 and args.mean_mode == "channel" and not args.paged
    ratios, why = traffic_ratios() if counters_cover else (None, "the counter runs covered the default format only")
    if ratios and all(b_ in ratios for b_ in bits):
        traffic = int(sum(st["layer_bytes"][l] * ratios[bits[l]] for l in range(L)) / L)
        traffic_source = "profiles/" + why
        for b_ in set(bits):
            per_bits[str(b_)]["traffic"] = int(per_bits[str(b_)]["bytes"] * ratios[b_])
    else:
        traffic_source = why

    # ---- the measured ceiling: the library's plain streaming read over buffers of the launches' sizes
    ceiling = stream_read_ceiling(env, {b_: v["bytes"] for b_, v in per_bits.items()})
    for b_ in per_bits:
        per_bits[b_]["frac_of_stream_read"] = round(per_bits[b_]["GBps"] / ceiling[b_], 4)
    c0, c1 = env.event_pair()

    # ---- context only: one layer of the same shape as a 16-bit cache, attended by torch's own
    # scaled_dot_product_attention (not tuned for decode) -- what the packed cache is an alternative to
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

    # ---- single-token append cost, measured apart from the timed region (real calls on spare capacity)
    torch.cuda.synchronize()
    app_t0 = time.perf_counter()
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
    # ---- single-token append: what a call costs the host, split into the binding's Python (tensor
    # slicing, checks, pointer extraction) and the library call itself, and what it costs the GPU
    n1 = 48
    host_split = {}
    for how in ("binding", "library"):
        kv.kv_cache_reset(scratch.handle, -1)
        torch.cuda.synchronize()
        c0.record(stream)
        t0 = time.perf_counter()
        if how == "binding":
            for i in range(n1):
                scratch.append(0, kr[:, i:i + 1], vr[:, i:i + 1])
        else:
            kp, vp, esz = kr.data_ptr(), vr.data_ptr(), kr.element_size()
            s0, s1, s2, sp_ = kr.stride(0), kr.stride(1), kr.stride(2), stream.cuda_stream
            for i in range(n1):
                kv.kv_quant_append(scratch.handle, 0, kp + i * s1 * esz, vp + i * s1 * esz, 1, s0, s1, s2, sp_)
        t_host = time.perf_counter() - t0  # the calls have returned; the GPU may still be busy
        c1.record(stream)
        c1.synchronize()
        host_split[how + "_host_us_per_call"] = round(t_host / n1 * 1e6, 2)
        host_split[how + "_gpu_us_per_call"] = round(c0.elapsed_time(c1) / n1 * 1e3, 2)
    host_split["python_marshalling_us_per_call"] = round(host_split["binding_host_us_per_call"] - host_split["library_host_us_per_call"], 2)
    host_split["note"] = ("one layer, batch %d, one token per sequence and call; host = wall time until the calls have returned "
                          "(enqueue only), gpu = event time over the same calls" % B)
    scratch.close()
    del scratch, kr, vr

    result = {
        "metric": "decode_attn_effective_hbm_GBps",
        "value": fig["value_GBps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": fig["ms_per_step"],
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
        "pct_of_hbm_peak": fig["pct_of_hbm_peak"],
        "decode_tokens_per_s": fig["decode_tokens_per_s"],
        "quant_append": {
            "bulk_tokens_per_s": fig["bulk_append_tokens_per_s"],
            "bulk_input_GBps": fig["bulk_append_input_GBps"],
            "single_token_tokens_per_s": round(B * n_app / app_s, 1) if n_app else None,
            "single_token_us_per_layer_call": round(app_s / max(n_app * L, 1) * 1e6, 2) if n_app else None,
            "single_token_call_cost": host_split,
            "bulk_4096_token_calls": rope_stats,
        },
        "roofline": {"bound": "hbm", "kernel": "decode split kernel (all layers, weighted by layer)",
                     "achieved": fig["split_kernels_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": fig["split_kernels_frac_of_peak"], "traffic": traffic, "traffic_source": traffic_source,
                     "bytes_per_launch": fig["bytes_per_launch"], "per_bits": per_bits,
                     "duration_source": "HIP events stamped by each split kernel's own dispatch (kv_time_next_split: begin and end "
                                        "of the kernel, as a kernel trace reports it), averaged over the timed steps",
                     "stream_read_GBps_same_size": ceiling,
                     "stream_read_kernel": "kv_stream_read_probe (read-only, 16-byte loads, one workgroup per contiguous 64 KiB)"},
        "context_16bit_cache": sdpa_ctx,
    }

    # ---- CPU oracle on a bounded sample of the same workload (rank 0): one thread, then one thread per (sequence, layer) task
    if NS and st["host_kv"]:
        result["cpu_baseline"] = cpu_baseline(env, st, NS, Hq, Hkv, G, T0, K, W, n_app)
    release(env, st)
    del cache, k_dec, q_dec

    # ---- the baseline's other configurations, a few seconds each
    legs = [] if args.legs == "none" else [x for x in args.legs.split(",") if x]
    other = {}
    ks, kw = args.leg_steps, 2
    for leg in legs:
        t_leg = time.perf_counter()
        try:
            if leg == "c0":
                other["config0_single_head"] = latency_leg(env, "config 0", Hq=1, Hkv=1, T=1024, dtype_name="fp16")
            elif leg == "c1":
                other["config1_llama8b_layer"] = latency_leg(env, "config 1", Hq=32, Hkv=8, T=8205, dtype_name="bf16")
            elif leg == "c3":
                f3, s3 = run_decode_workload(env, L=80, B=1, Hq=64, Hkv=8, G=64, T0=131072, steps=ks, warmup=kw,
                                             scheme="mixed24_8ends", seed=3000, shared_inputs=True, chunk=16384)
                f3["workload"] = "config 3: 80 layers, batch 1, 64q/8kv heads, context 131072, bf16, G=Gc=64, mixed 2/4-bit map with 8-bit first and last two layers (seed 3000)"
                # the same steps replayed from one HIP graph (a layer is one launch of 30-60 us on 8 units there)
                f3["graph_replay"] = graph_leg(env, f3, s3)
                other["config3_long_context"] = f3
                release(env, s3)
            elif leg == "c4":
                f4, s4 = run_decode_workload(env, L=32, B=64, Hq=32, Hkv=8, G=32, T0=16384, steps=ks, warmup=kw,
                                             scheme="mixed248", seed=4000, shared_inputs=True, chunk=1024)
                f4["workload"] = ("config 4: 32 layers, batch 64, 32q/8kv heads, bf16, G=Gc=32, mixed 2/4/8-bit map (seed 4000): bulk quantise-append of a "
                                  "16384-token prefill in 1024-token calls, then decode steps (append + attend); %d of the 512 steps timed" % ks)
                other["config4_prefill_then_decode"] = f4
                release(env, s4)
            elif leg == "cross":
                fx, sx = run_decode_workload(env, L=8, B=16, Hq=32, Hkv=8, G=32, T0=32768, steps=ks, warmup=kw,
                                             scheme="mixed248", seed=2000, mean_mode="cross", shared_inputs=True)
                fx["workload"] = "headline shape with the mean over the kv heads (Eq. 1-2): first 8 layers of the bit map, batch 16, context 32768"
                # the same steps replayed from one HIP graph (four launches per layer: the mean rows of a block about to be compressed first)
                fx["graph_replay"] = graph_leg(env, fx, sx, launches=4)
                other["cross_head_mean"] = fx
                release(env, sx)
            elif leg == "cross128":
                fy, sy = run_decode_workload(env, L=8, B=16, Hq=32, Hkv=8, G=128, T0=32768, steps=ks, warmup=kw,
                                             scheme="mixed248", seed=2000, mean_mode="cross", shared_inputs=True)
                fy["workload"] = ("headline shape with the mean over the kv heads and groups of 128 (the format of the paper's Sec. 3 "
                                  "storage example): first 8 layers of the bit map, batch 16, context 32768")
                other["cross_head_mean_groups_of_128"] = fy
                release(env, sy)
            elif leg == "mixed":
                fm, sm = run_decode_workload(env, L=8, B=16, Hq=32, Hkv=8, G=32, Gc=128, T0=32768, steps=ks, warmup=kw,
                                             scheme="mixed248", seed=2000, shared_inputs=True)
                fm["workload"] = ("headline shape with key groups of 32 tokens and one value group per token (G = 32, Gc = 128): "
                                  "first 8 layers of the bit map, batch 16, context 32768")
                other["mixed_group_sizes"] = fm
                release(env, sm)
            elif leg == "widths":
                fw, sw = run_decode_workload(env, L=8, B=16, Hq=32, Hkv=8, G=32, T0=32768, steps=ks, warmup=kw, v_bits=(4, 2),
                                             scheme="mixed248", seed=2000, shared_inputs=True)
                fw["workload"] = "headline shape with 4-bit keys and 2-bit values in all of 8 layers, batch 16, context 32768"
                other["different_widths_k4_v2"] = fw
                release(env, sw)
            elif leg == "graph":
                # the headline shape's first 8 layers and the batch-1 long context, eager and replayed
                fg, sg = run_decode_workload(env, L=8, B=16, Hq=32, Hkv=8, G=32, T0=32768, steps=ks, warmup=kw,
                                             scheme="mixed248", seed=2000, shared_inputs=True)
                other["graph_replay_headline_shape"] = graph_leg(env, fg, sg)
                release(env, sg)
            elif leg == "compressv":
                other["compressv_config2_shape"] = compressv_leg(env, B=16, n=4096)
                other["compressv_config4_shape"] = compressv_leg(env, B=64, n=1024)
            else:
                other[leg] = {"error": "unknown leg"}
                continue
        except Exception as ex:  # a leg that fails leaves the headline line valid
            other[leg] = {"error": repr(ex)[:200]}
            torch.cuda.empty_cache()
        for key in other:
            if isinstance(other[key], dict) and "leg_wall_s" not in other[key]:
                other[key]["leg_wall_s"] = round(time.perf_counter() - t_leg, 1)
    if other:
        result["other_configs"] = other
    print(json.dumps(result))


def cpu_baseline(env, st, NS, Hq, Hkv, G, T0, K, W, n_app):
    import concurrent.futures as cf

    import oracle

    np, torch, kv = env.np, env.torch, env.kv
    cache, k_dec, q_dec, sample_layers = st["cache"], st["k_dec"], st["q_dec"], st["sample_layers"]
    d = 128
    ocfg_bits = [sample_layers[l] for l in sorted(sample_layers)]
    nl = len(ocfg_bits)
    B = cache.cfg.batch

    def u16(t):
        return t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

    def make(ns):
        return oracle.OracleCache(oracle.OracleConfig(nl, ns, Hq, Hkv, d, st["max_tokens"], G, G, st["R"], oracle.tada.BF16,
                                                      st["mm"], ocfg_bits, ocfg_bits))

    def replay(orc, i, l, lo, hi):
        kd, vd = k_dec[l]
        for s in list(range(W + K)) + list(range(n_app)):
            orc.append(i, u16(kd[lo:hi, s:s + 1]), u16(vd[lo:hi, s:s + 1]))

    # one thread: all NS sequences in one oracle cache
    orc = make(NS)
    enc_s = att_s = 0.0
    att_bytes = 0
    worst = 0.0
    for i, l in enumerate(sorted(sample_layers)):
        hk, hv = st["host_kv"][l]
        k16, v16 = u16(hk), u16(hv)
        t0 = time.perf_counter()
        orc.append(i, k16, v16)
        enc_s += time.perf_counter() - t0
        replay(orc, i, l, 0, NS)  # the decode tokens that the GPU cache has seen, so both hold the same state
        q16 = u16(q_dec[l][0:NS])
        t0 = time.perf_counter()
        want = orc.attend(i, q16)
        att_s += time.perf_counter() - t0
        got = cache.attend(l, q_dec[l])
        torch.cuda.synchronize()
        worst = max(worst, float(np.max(np.abs(got[0:NS].cpu().numpy().astype(np.float64) - want))))
        att_bytes += kv.kv_decode_bytes(cache.handle, l) * NS // B
    del orc

    # one thread per (sequence, layer) of the sample, as many at a time as the host has cores (the oracle's C
    # routines release the interpreter lock); every task has an oracle cache of its own
    def one_task(task):
        b, i, l = task
        o = oracle.OracleCache(oracle.OracleConfig(1, 1, Hq, Hkv, d, st["max_tokens"], G, G, st["R"], oracle.tada.BF16,
                                                   st["mm"], [ocfg_bits[i]], [ocfg_bits[i]]))
        hk, hv = st["host_kv"][l]
        t0 = time.perf_counter()
        o.append(0, u16(hk[b:b + 1]), u16(hv[b:b + 1]))
        te = time.perf_counter() - t0
        replay(o, 0, l, b, b + 1)
        t0 = time.perf_counter()
        o.attend(0, u16(q_dec[l][b:b + 1]))
        return te, time.perf_counter() - t0

    tasks = [(b, i, l) for b in range(NS) for i, l in enumerate(sorted(sample_layers))]
    threads = min(len(tasks), os.cpu_count() or 1)
    t0 = time.perf_counter()
    with cf.ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(one_task, tasks))
    par_wall = time.perf_counter() - t0
    par_busy = sum(a + b for a, b in parts)
    return {
        "value": round(att_bytes / att_s / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": "batch elements 0-%d (%d kv-head units, full context) of one layer per bit width %s: "
                  "decode attention %.2f s; their quantise-append %.2f s = %.0f tokens/s"
                  % (NS - 1, NS * Hkv, ocfg_bits, att_s, enc_s, nl * NS * T0 / enc_s),
        "quant_append_tokens_per_s": round(nl * NS * T0 / enc_s, 1),
        "gpu_vs_oracle_max_abs_err": worst,
        "host_cpu_count": os.cpu_count(),
        "threaded": {"cores": threads, "wall_s": round(par_wall, 2), "sum_of_thread_times_s": round(par_busy, 2),
                     "value": round(att_bytes / (par_wall * att_s / max(att_s + enc_s, 1e-9)) / 1e9, 4), "unit": "GB/s",
                     "note": "the same sample as one task per (sequence, layer), append + attention per task, one thread per "
                             "task up to the host's core count; value = decode bytes / the wall time's attention share"},
    }


if __name__ == "__main__":
    main()
