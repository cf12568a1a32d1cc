"""Pins for the CPU oracle's empirical caching policies (Sec. 3.2: "sim." counts accesses over
simulated epochs, "oracle" over the evaluated ones; both are ranked like a VIP score)."""
import numpy as np
import pytest

import oracle
from workloads import synth as S


def test_count_against_library_histogram():
    rng = np.random.default_rng(2)
    N = 500
    count = None
    want = np.zeros(N)
    for _ in range(5):
        ids = rng.integers(0, N, size=300).astype(np.int32)
        count = oracle.access_count(N, ids, count)
        want += np.bincount(ids, minlength=N)
    assert np.array_equal(count, want.astype(np.float32))
    assert oracle.access_count(N, []).sum() == 0
    with pytest.raises(ValueError):
        oracle.access_count(N, [3, N])
    with pytest.raises(ValueError):
        oracle.access_count(N, [-1])


def _epoch_counts(cfg, g, Tk, epochs, seed, B=None, fanouts=None):
    B = B or cfg.B
    fanouts = fanouts or cfg.fanouts
    rowptr, col = g.rowptr.numpy(), g.col.numpy()
    count = np.zeros(g.N, dtype=np.float32)
    nb = 0
    for ep in epochs:
        perm = np.random.default_rng(1000 + ep).permutation(Tk.numpy())
        for b in range(0, perm.size - B + 1, B):
            m = oracle.sample_mfg(rowptr, col, perm[b:b + B], fanouts, seed, ep * 1000 + b // B)
            assert np.unique(m.node_ids).size == m.node_ids.size        # at most +1 per minibatch
            oracle.access_count(g.N, m.node_ids, count)
            nb += 1
    return count, nb


def test_counts_bounded_by_minibatches_and_seeds_counted_once_per_epoch(tiny):
    cfg, g, T, Tk = tiny
    count, nb = _epoch_counts(cfg, g, Tk, [0, 1], 7, B=64, fanouts=(5, 5))
    assert count.max() <= nb
    # every training vertex that fell into a full minibatch is a seed exactly once per epoch, so it is counted at least
    # (epochs it was a seed in) times; at most 63 vertices per epoch are left over
    assert (count[Tk.numpy()] >= 1).sum() >= Tk.numel() - 63


def test_empirical_frequency_approaches_vip_and_retroactive_ranking_is_optimal(tiny):
    """The count over many minibatches divided by their number estimates the inclusion probability
    (Sec. 3.1), and for a fixed cache size the retroactive ranking leaves the fewest misses on the
    epochs it was made from: no other set of that size, in particular the VIP-ranked and the
    simulated one, can miss less (Sec. 3.2, the lower bound of the policy comparison)."""
    cfg, g, T, Tk = tiny
    lo, hi = cfg.bounds()
    B, fanouts = 64, (5, 5)
    pt, _ = oracle.vip(g.rowptr.numpy(), g.col.numpy(), Tk.numpy(), B, fanouts)
    sim, nb_sim = _epoch_counts(cfg, g, Tk, [100, 101], 7, B, fanouts)
    ev, nb_ev = _epoch_counts(cfg, g, Tk, list(range(12)), 7, B, fanouts)
    remote = np.ones(g.N, bool)
    remote[lo:hi] = False
    # frequencies against probabilities, vertex by vertex: within 5 binomial standard deviations (+ the model's own
    # approximation, which is small on this graph) for all but a handful of vertices, and nearly unbiased in total
    # (S_L holds the seeds too, so the hop-0 term is multiplied in for this comparison)
    p_all, _ = oracle.vip(g.rowptr.numpy(), g.col.numpy(), Tk.numpy(), B, fanouts, include_hop0=True)
    freq = ev / nb_ev
    sd = np.sqrt(np.maximum(p_all * (1 - p_all), 1e-12) / nb_ev)
    off = np.abs(freq - p_all) > 5 * sd + 0.02
    assert off.mean() < 0.005
    # (the sampler expands all of S_{h-1} at hop h, the printed model only the vertices of hop h-1: the
    # model's total is a few per cent low)
    assert abs(freq[remote].sum() - pt[remote].sum()) < 0.05 * pt[remote].sum()
    total = ev[remote].sum()
    for alpha in (0.05, 0.2):
        misses = {}
        for name, score in (("vip", pt.astype(np.float32)), ("sim", sim), ("oracle", ev)):
            ids = oracle.cache_select(score, lo, hi, cfg.K, alpha)
            misses[name] = total - ev[ids].sum()
        assert misses["oracle"] <= misses["vip"] and misses["oracle"] <= misses["sim"]
        # the analytic model is close to the retroactive bound, and no worse than two simulated epochs by more than noise
        assert misses["vip"] <= 1.10 * misses["oracle"]
        assert misses["vip"] <= 1.02 * misses["sim"]
        # brute force on a random alternative of the same size
        c = oracle.cache_capacity(g.N, cfg.K, alpha)
        alt = np.random.default_rng(0).choice(np.flatnonzero(remote), size=c, replace=False)
        assert total - ev[alt].sum() >= misses["oracle"]
