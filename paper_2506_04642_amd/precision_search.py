"""Per-layer quantisation precision search on a synthetic proxy (arxiv 2506.04642, Sec. 3.3
"Searching for quantization precision", App. B).

The paper picks one width in {2, 4, 8} per layer by random search, scoring candidates on a small
sample of training data.  Model weights and datasets are not available here, so the score is a
proxy measured on the HIP path itself: for every layer a seeded synthetic cache is stored at each
candidate width and at 16 bits, and the error of the decode-attention output against the 16-bit
cache is the layer's cost at that width.  The search then draws random bit maps, keeps those whose
cache size stays within a byte budget (fraction of the 16-bit cache, as in the paper's 27 %), and
returns the one with the smallest summed cost.  Because the proxy treats layers independently the
exact optimum is also available (a multiple-choice knapsack), and `search` reports how close the
random search came.

`measure_layer_errors` needs the GPU; `random_search` and `exact_optimum` are host arithmetic on
its table and run anywhere.
"""
from __future__ import annotations

from typing import Dict, Sequence, Tuple

import numpy as np

WIDTHS = (2, 4, 8)


def bytes_per_token(head_dim: int, group_tokens: int, group_channels: int, mean_mode: int = 0,
                    n_kv_heads: int = 8) -> Dict[int, float]:
    """Stored bytes per (kv head, token) at each width, metadata included (16 -> raw).  Mirrors the
    record of the storage format: codes for K and V, K scale/zero per channel and block, V scale/zero
    per token and channel group, and the mean: one binary16 value per channel and block for K and
    for V (per-channel block mean), or a kv head's share of the two binary16 mean vectors per
    token (mean over the kv heads, Eq. 1-2)."""
    d, G, Gc = head_dim, group_tokens, group_channels
    out = {16: 2.0 * d * 2}
    for b in WIDTHS:
        codes = 2.0 * d * b / 8
        meta = 2 * 2.0 * d / G + 2 * 2.0 * d / Gc
        mean = 2 * 2.0 * d / G if mean_mode == 0 else (2 * 2.0 * d / n_kv_heads if mean_mode == 1 else 0.0)
        out[b] = codes + meta + mean
    return out


def layer_recipe(seed: int, layer: int, n_layers: int) -> Tuple[int, float]:
    """Synthetic stand-in for 'sensitivity varies across layers': the number of outlier channels
    and the query temperature of a layer, drawn once per (seed, layer)."""
    rng = np.random.default_rng([seed, layer, 77])
    n_outlier = int(rng.integers(2, 9))
    temperature = float(rng.uniform(0.5, 1.5)) * (1.0 + 0.5 * (n_layers - 1 - layer) / max(n_layers - 1, 1))
    return n_outlier, temperature


def measure_layer_errors(n_layers: int, *, seed: int = 0, batch: int = 2, n_q_heads: int = 8, n_kv_heads: int = 2,
                         context: int = 1024, group: int = 32, dtype: int = 1, mean_mode: int = 0,
                         shared_sigma: float = 0.0, device: str = "cuda:0") -> np.ndarray:
    """err[l, i]: root-mean-square error of the decode-attention output of layer l stored at
    WIDTHS[i] against the same layer stored at 16 bits, relative to the rms of that output.
    Everything runs through the C ABI (quantise-append, decode attention)."""
    import torch

    from . import binding as kv
    from . import synth

    d = 128
    bits = list(WIDTHS) + [16]
    cfg = kv.make_config(len(bits), batch, n_q_heads, n_kv_heads, d, context + group, group, group, group, dtype,
                         mean_mode, bits, bits)
    cache = kv.KVCache(cfg, device=device, zero=False)
    err = np.zeros((n_layers, len(WIDTHS)))
    for l in range(n_layers):
        n_outlier, temperature = layer_recipe(seed, l, n_layers)
        k, v = synth.make_kv_torch(seed * 1000 + l, batch, context, n_kv_heads, d, dtype, device, n_outlier=n_outlier,
                                   shared_sigma=shared_sigma)
        q = synth.make_q_torch(seed * 1000 + l, batch, n_q_heads, d, dtype, device)
        q = (q.float() * temperature).to(q.dtype)
        kv.kv_cache_reset(cache.handle, -1)
        outs = []
        for i in range(len(bits)):
            cache.append(i, k, v)
            outs.append(cache.attend(i, q).double())
        ref = outs[-1]
        scale = float(ref.pow(2).mean().sqrt())
        for i in range(len(WIDTHS)):
            err[l, i] = float((outs[i] - ref).pow(2).mean().sqrt()) / scale
    cache.close()
    return err


def measure_reconstruction_errors(n_layers: int, *, seed: int = 0, batch: int = 2, n_q_heads: int = 8, n_kv_heads: int = 2,
                                  context: int = 1024, group: int = 32, dtype: int = 1, mean_mode: int = 0,
                                  shared_sigma: float = 0.0, device: str = "cuda:0") -> np.ndarray:
    """err[l, i, side]: Frobenius norm of (x - x^) over that of x for the keys (side 0) and values
    (side 1) of synthetic layer l stored at WIDTHS[i]; x^ is the cache's reconstruction (Eq. 7-8)
    through the C ABI."""
    import torch

    from . import binding as kv
    from . import synth

    d = 128
    bits = list(WIDTHS)
    cfg = kv.make_config(len(bits), batch, n_q_heads, n_kv_heads, d, context + group, group, group, group, dtype,
                         mean_mode, bits, bits)
    cache = kv.KVCache(cfg, device=device, zero=False)
    err = np.zeros((n_layers, len(WIDTHS), 2))
    for l in range(n_layers):
        n_outlier, _ = layer_recipe(seed, l, n_layers)
        k, v = synth.make_kv_torch(seed * 1000 + l, batch, context, n_kv_heads, d, dtype, device, n_outlier=n_outlier,
                                   shared_sigma=shared_sigma)
        kv.kv_cache_reset(cache.handle, -1)
        for i in range(len(bits)):
            cache.append(i, k, v)
            kh, vh = cache.dequant(i, context)
            for side, (x, xh) in enumerate(((k, kh), (v, vh))):
                x = x.double()
                err[l, i, side] = float((x - xh.double()).pow(2).sum().sqrt() / x.pow(2).sum().sqrt())
    cache.close()
    return err


def mean_mode_table(n_layers: int = 4, *, seed: int = 0, shared_sigma: float = 2.0, **measure_kw) -> Dict[str, list]:
    """Synthetic analogue of the paper's error comparison with and without mean-centring (Fig. 2):
    the relative Frobenius error of the reconstructed keys and values and the decode-attention
    error against the 16-bit cache, averaged over n_layers synthetic layers,
    for no mean, the per-channel block mean and the mean over kv heads, at 2 / 4 / 8 bits.  The
    inputs carry a component shared by all kv heads (shared_sigma), which is the structure the
    paper attributes to real caches; with shared_sigma = 0 the mean over heads has nothing to
    remove."""
    out = {}
    measure_kw.setdefault("n_kv_heads", 8)
    measure_kw.setdefault("n_q_heads", 32)
    group = measure_kw.get("group", 32)
    for name, mode in (("none", 2), ("channel_block", 0), ("cross_head", 1)):
        err = measure_layer_errors(n_layers, seed=seed, mean_mode=mode, shared_sigma=shared_sigma, **measure_kw)
        per_token = bytes_per_token(128, group, group, mode, measure_kw["n_kv_heads"])
        rec = measure_reconstruction_errors(n_layers, seed=seed, mean_mode=mode, shared_sigma=shared_sigma, **measure_kw)
        out[name] = {"rel_rms_error": [float(x) for x in err.mean(axis=0)],
                     "k_rel_frobenius": [float(x) for x in rec[:, :, 0].mean(axis=0)],
                     "v_rel_frobenius": [float(x) for x in rec[:, :, 1].mean(axis=0)],
                     "bytes_vs_16bit": [per_token[b] / per_token[16] for b in WIDTHS]}
    return out


def map_cost(err: np.ndarray, bit_map: Sequence[int]) -> float:
    return float(sum(err[l, WIDTHS.index(b)] for l, b in enumerate(bit_map)))


def map_ratio(bit_map: Sequence[int], per_token: Dict[int, float]) -> float:
    """Cache size of the map relative to the 16-bit cache."""
    return float(sum(per_token[b] for b in bit_map) / (len(bit_map) * per_token[16]))


def random_search(err: np.ndarray, per_token: Dict[int, float], budget: float, *, n_candidates: int = 20000,
                  seed: int = 0) -> Tuple[list, float]:
    """Random search as in the paper: draw bit maps, drop those over the byte budget, keep the one
    with the smallest summed proxy error.  Candidates are drawn with a per-candidate mix of the
    three widths so that all cache sizes are visited.  Returns (bit map, cost); the all-2-bit map
    is the fallback if it alone fits, ValueError if nothing fits."""
    L = err.shape[0]
    rng = np.random.default_rng(seed)
    best, best_cost = None, np.inf
    floor = [WIDTHS[0]] * L
    if map_ratio(floor, per_token) <= budget:
        best, best_cost = floor, map_cost(err, floor)
    widths = np.array(WIDTHS)
    sizes = np.array([per_token[b] for b in WIDTHS])
    limit = budget * L * per_token[16]
    for _ in range(n_candidates):
        p = rng.dirichlet(np.ones(len(WIDTHS)))
        idx = rng.choice(len(WIDTHS), size=L, p=p)
        if sizes[idx].sum() > limit:
            continue
        cost = float(err[np.arange(L), idx].sum())
        if cost < best_cost:
            best, best_cost = [int(b) for b in widths[idx]], cost
    if best is None:
        raise ValueError("no bit map fits the budget")
    return best, best_cost


def exact_optimum(err: np.ndarray, per_token: Dict[int, float], budget: float) -> Tuple[list, float]:
    """Smallest summed proxy error under the byte budget (layers are independent in the proxy, so
    this is a multiple-choice knapsack; sizes are multiples of a common unit of bytes)."""
    L = err.shape[0]
    unit = 0.5
    sizes = [int(round(per_token[b] / unit)) for b in WIDTHS]
    cap = int(np.floor(budget * L * per_token[16] / unit + 1e-9))
    INF = float("inf")
    best = np.full(cap + 1, INF)
    best[0] = 0.0
    choice = np.zeros((L, cap + 1), dtype=np.int8)
    for l in range(L):
        nxt = np.full(cap + 1, INF)
        for i, sz in enumerate(sizes):
            if sz > cap:
                continue
            cand = np.full(cap + 1, INF)
            cand[sz:] = best[: cap + 1 - sz] + err[l, i]
            better = cand < nxt
            nxt[better] = cand[better]
            choice[l][better] = i
        best = nxt
    end = int(np.argmin(best))
    if not np.isfinite(best[end]):
        raise ValueError("no bit map fits the budget")
    bit_map, c = [], end
    for l in range(L - 1, -1, -1):
        i = int(choice[l][c])
        bit_map.append(WIDTHS[i])
        c -= sizes[i]
    return bit_map[::-1], float(best[end])


def search(n_layers: int, budget: float = 0.27, *, seed: int = 0, n_candidates: int = 20000, **measure_kw) -> dict:
    """Measure the proxy on the GPU, run the random search, and report it next to the exact optimum."""
    err = measure_layer_errors(n_layers, seed=seed, **measure_kw)
    group = measure_kw.get("group", 32)
    per_token = bytes_per_token(128, group, group, measure_kw.get("mean_mode", 0))
    found, cost = random_search(err, per_token, budget, n_candidates=n_candidates, seed=seed)
    opt, opt_cost = exact_optimum(err, per_token, budget)
    return {"bit_map": found, "cost": cost, "ratio": map_ratio(found, per_token), "optimum": opt,
            "optimum_cost": opt_cost, "errors": err}


if __name__ == "__main__":
    import argparse
    import json

    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--budget", type=float, default=0.27, help="cache bytes as a fraction of the 16-bit cache")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--candidates", type=int, default=20000)
    ap.add_argument("--mean-modes", action="store_true",
                    help="print the error table over mean modes and widths instead of searching")
    ap.add_argument("--shared-sigma", type=float, default=2.0, help="component common to all kv heads (--mean-modes)")
    ap.add_argument("--group", type=int, default=32, choices=[32, 64, 128], help="group size G = Gc (--mean-modes)")
    a = ap.parse_args()
    if a.mean_modes:
        print(json.dumps({"widths": list(WIDTHS), "group": a.group,
                          "mean_modes": mean_mode_table(min(a.layers, 8), seed=a.seed, shared_sigma=a.shared_sigma,
                                                        group=a.group)}))
        raise SystemExit(0)
    r = search(a.layers, a.budget, seed=a.seed, n_candidates=a.candidates)
    r["errors"] = np.round(r["errors"], 5).tolist()
    print(json.dumps(r))
