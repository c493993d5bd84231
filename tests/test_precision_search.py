"""Precision search (Sec. 3.3, App. B): host logic on the CPU, the measured proxy on the GPU."""
import itertools

import numpy as np
import pytest

from paper_2506_04642_amd import precision_search as ps
from paper_2506_04642_amd import synth


def _table(seed, L):
    rng = np.random.default_rng(seed)
    e8 = rng.uniform(0.001, 0.01, L)
    e4 = e8 * rng.uniform(4, 20, L)
    e2 = e4 * rng.uniform(2, 10, L)
    return np.stack([e2, e4, e8], axis=1)


def test_bytes_per_token_match_the_storage_format():
    pt = ps.bytes_per_token(128, 32, 32, 0)
    assert (pt[2], pt[4], pt[8], pt[16]) == (112.0, 176.0, 304.0, 512.0)
    pt = ps.bytes_per_token(128, 64, 64, 0)
    assert (pt[2], pt[4], pt[8]) == (88.0, 152.0, 280.0)
    # 24 layers at 4 bits and 8 at 2 bits: the mix the paper reports at 0.27 of the 16-bit cache
    # (Tables 1, 2 and 5; its own metadata accounting differs slightly from this format's)
    ratio = ps.map_ratio([4] * 24 + [2] * 8, ps.bytes_per_token(128, 32, 32, 0))
    assert abs(ratio - 0.3125) < 1e-12 and 0.25 < ratio < 0.35


def test_bytes_per_token_cross_head_mean_matches_the_paper_formula():
    """Sec. 3 memory formula: at 4 bits, 8 kv heads and groups of 32 the cache is
    1/8 + 4/16 + 2/32 = 43.75 % of the 16-bit cache."""
    pt = ps.bytes_per_token(128, 32, 32, 1, n_kv_heads=8)
    assert pt[4] / pt[16] == 1 / 8 + 4 / 16 + 2 / 32


@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("budget", [0.23, 0.27, 0.4, 0.6])
def test_exact_optimum_equals_brute_force(seed, budget):
    L = 6
    err, pt = _table(seed, L), ps.bytes_per_token(128, 32, 32, 0)
    best = min((ps.map_cost(err, m) for m in itertools.product(ps.WIDTHS, repeat=L) if ps.map_ratio(m, pt) <= budget))
    m, c = ps.exact_optimum(err, pt, budget)
    assert ps.map_ratio(m, pt) <= budget + 1e-12
    assert abs(c - best) < 1e-12 and abs(ps.map_cost(err, m) - c) < 1e-12


def test_random_search_respects_the_budget_and_approaches_the_optimum():
    L = 32
    err, pt = _table(7, L), ps.bytes_per_token(128, 32, 32, 0)
    prev = np.inf
    for budget in (0.22, 0.27, 0.35, 0.5):
        m, c = ps.random_search(err, pt, budget, n_candidates=20000, seed=1)
        assert len(m) == L and set(m) <= set(ps.WIDTHS)
        assert ps.map_ratio(m, pt) <= budget + 1e-12
        _, opt = ps.exact_optimum(err, pt, budget)
        assert opt - 1e-12 <= c <= max(2.5 * opt, opt + 0.5)
        assert c <= prev + 1e-12  # a larger budget never costs more (same candidate stream)
        prev = c
    few, c_few = ps.random_search(err, pt, 0.27, n_candidates=50, seed=1)
    many, c_many = ps.random_search(err, pt, 0.27, n_candidates=5000, seed=1)
    assert c_many <= c_few
    with pytest.raises(ValueError):
        ps.random_search(err, pt, 0.1)
    with pytest.raises(ValueError):
        ps.exact_optimum(err, pt, 0.1)


@pytest.mark.gpu
def test_measured_proxy_matches_the_oracle(oracle):
    import torch

    L, B, Hq, Hkv, T, G = 3, 2, 8, 2, 256, 32
    got = ps.measure_layer_errors(L, seed=5, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, context=T, group=G, dtype=1)
    assert np.all(got[:, 0] > got[:, 1]) and np.all(got[:, 1] > got[:, 2]) and np.all(got[:, 2] > 0)
    want = np.zeros_like(got)
    for l in range(L):
        n_outlier, temperature = ps.layer_recipe(5, l, L)
        k, v = synth.make_kv_torch(5000 + l, B, T, Hkv, 128, 1, "cuda:0", n_outlier=n_outlier)
        q = synth.make_q_torch(5000 + l, B, Hq, 128, 1, "cuda:0")
        q = (q.float() * temperature).to(q.dtype)
        kb, vb, qb = (t.cpu().view(torch.int16).numpy().view(np.uint16) for t in (k, v, q))
        bits = [2, 4, 8, 16]
        cfg = oracle.OracleConfig(4, B, Hq, Hkv, 128, T + G, G, G, G, 1, 0, bits, bits)
        orc = oracle.OracleCache(cfg)
        outs = []
        for i in range(4):
            orc.append(i, kb, vb)
            outs.append(orc.attend(i, qb))
        scale = np.sqrt(np.mean(outs[3] ** 2))
        for i in range(3):
            want[l, i] = np.sqrt(np.mean((outs[i] - outs[3]) ** 2)) / scale
    assert np.allclose(got, want, rtol=1e-3, atol=1e-5), (got, want)


@pytest.mark.gpu
def test_mean_over_heads_removes_a_shared_component():
    """Synthetic analogue of the paper's error comparison (Fig. 2): with a component common to
    all kv heads the mean over heads cuts the attention error at every width; without one the
    deviations only lose the 1/H of the variance that the mean carries."""
    import torch

    assert torch.cuda.is_available(), "needs the GPU"
    print("case mean_mode_table", flush=True)
    shared = ps.mean_mode_table(2, seed=3, shared_sigma=2.0, context=512)
    plain = ps.mean_mode_table(2, seed=3, shared_sigma=0.0, context=512)
    for i in range(3):
        assert shared["cross_head"]["rel_rms_error"][i] < 0.6 * shared["none"]["rel_rms_error"][i]
        r = plain["cross_head"]["rel_rms_error"][i] / plain["none"]["rel_rms_error"][i]
        assert 0.75 < r < 1.05
    assert shared["cross_head"]["bytes_vs_16bit"][1] == 0.4375
