"""Pins for the CPU oracle's cache ranking (Sec. 3.2) and cache-aware gather (Secs. 4.1-4.3)."""
import numpy as np
import pytest
import torch

import oracle
from workloads import synth as S


def _scores(tiny):
    cfg, g, T, Tk = tiny
    pt, _ = oracle.vip(g.rowptr.numpy(), g.col.numpy(), Tk.numpy(), cfg.B, cfg.fanouts)
    return pt.astype(np.float32)


def test_capacity_is_floor_alpha_n_over_k():
    assert oracle.cache_capacity(10_000, 4, 0.10) == 250
    assert oracle.cache_capacity(111_000_000, 8, 0.32) == 4_440_000
    assert oracle.cache_capacity(10, 4, 0.5) == 1          # floor(1.25)
    assert oracle.cache_capacity(10, 4, 0.0) == 0


def test_ranking_against_library_sort(tiny):
    cfg, g, T, Tk = tiny
    score = _scores(tiny)
    lo, hi = cfg.bounds()
    ids = oracle.cache_select(score, lo, hi, cfg.K, cfg.alpha)
    cand = np.flatnonzero((score > 0) & ~((np.arange(g.N) >= lo) & (np.arange(g.N) < hi)))
    order = np.lexsort((cand, -score[cand].astype(np.float64)))     # score desc, id asc
    want = cand[order][:cfg.cache_capacity()]
    assert np.array_equal(ids, want)
    assert ids.size <= cfg.cache_capacity()
    assert np.all((ids < lo) | (ids >= hi)) and np.all(score[ids] > 0)


def test_prefix_property_and_ties(tiny):
    cfg, g, T, Tk = tiny
    score = _scores(tiny)
    lo, hi = cfg.bounds()
    big = oracle.cache_select(score, lo, hi, cfg.K, 0.5)
    for a in (0.0, 0.05, 0.1, 0.2):
        small = oracle.cache_select(score, lo, hi, cfg.K, a)
        assert np.array_equal(small, big[:small.size])
    # heavy ties: a constant score keeps the lowest remote ids
    flat = np.ones(g.N, dtype=np.float32)
    ids = oracle.cache_select(flat, lo, hi, cfg.K, 0.02)
    assert np.array_equal(ids, np.arange(hi, hi + 50))
    # fewer positive candidates than capacity
    few = np.zeros(g.N, dtype=np.float32)
    few[[hi + 5, hi + 1, 3]] = [0.5, 0.7, 0.9]     # 3 is local (lo = 0): never cached
    assert oracle.cache_select(few, lo, hi, cfg.K, 0.1).tolist() == [hi + 1, hi + 5]


def test_selected_set_minimises_expected_misses(tiny):
    """For a fixed size the kept set maximises the kept probability mass (Sec. 3.2): swapping any
    member for any non-member cannot raise it."""
    cfg, g, T, Tk = tiny
    score = _scores(tiny)
    lo, hi = cfg.bounds()
    ids = oracle.cache_select(score, lo, hi, cfg.K, 0.05)
    remote = np.ones(g.N, bool)
    remote[lo:hi] = False
    inside = np.zeros(g.N, bool)
    inside[ids] = True
    assert score[ids].min() >= score[remote & ~inside].max()


def test_gather_rows_by_regeneration_and_counts(tiny):
    cfg, g, T, Tk = tiny
    lo, hi = cfg.bounds()
    score = _scores(tiny)
    cache_ids = oracle.cache_select(score, lo, hi, cfg.K, cfg.alpha)
    local = S.feature_block(cfg, lo, hi).numpy()
    remote = S.feature_rows(cfg, S.remote_ids(cfg, 0, cfg.N - (hi - lo))).numpy()
    cache_rows = S.feature_rows(cfg, torch.from_numpy(cache_ids)).numpy()
    seeds = S.epoch_batches(cfg, Tk, 0)[0].numpy()
    m = oracle.sample_mfg(g.rowptr.numpy(), g.col.numpy(), seeds, cfg.fanouts, cfg.seed_sampler, 0)
    out, tag, counts = oracle.gather(g.N, lo, hi, local, cache_rows, cache_ids, remote, m.node_ids)
    want = S.feature_rows(cfg, torch.from_numpy(m.node_ids)).numpy()
    assert np.array_equal(out.view(np.uint32), want.view(np.uint32))
    is_local = (m.node_ids >= lo) & (m.node_ids < hi)
    is_cached = np.isin(m.node_ids, cache_ids)
    assert counts == (int(is_local.sum()), int(is_cached.sum()), int((~is_local & ~is_cached).sum()))
    assert np.array_equal(tag == 0, is_local) and np.array_equal(tag == 1, is_cached)
    # a wrong cache row would show: poison the cache and see exactly the cached rows change
    bad = cache_rows.copy()
    bad += 1.0
    out2, _, _ = oracle.gather(g.N, lo, hi, local, bad, cache_ids, remote, m.node_ids)
    changed = np.any(out2 != out, axis=1)
    assert np.array_equal(changed, is_cached)
    # no cache at all (alpha = 0) and duplicate ids
    out3, tag3, c3 = oracle.gather(g.N, lo, hi, local, None, None, remote, [5, hi + 5, 5])
    assert c3 == (2, 0, 1) and np.array_equal(out3[0], out3[2])
    assert np.array_equal(out3, S.feature_rows(cfg, torch.tensor([5, hi + 5, 5])).numpy())


def test_hit_rate_grows_with_alpha(tiny):
    cfg, g, T, Tk = tiny
    lo, hi = cfg.bounds()
    score = _scores(tiny)
    seeds = S.epoch_batches(cfg, Tk, 0)[0].numpy()
    m = oracle.sample_mfg(g.rowptr.numpy(), g.col.numpy(), seeds, cfg.fanouts, cfg.seed_sampler, 0)
    prev = -1
    for a in (0.0, 0.05, 0.1, 0.2, 0.5):
        ids = oracle.cache_select(score, lo, hi, cfg.K, a)
        hits = int(np.isin(m.node_ids, ids).sum())
        assert hits >= prev
        prev = hits


def test_feature_rows_do_not_depend_on_the_request(tiny):
    cfg = tiny[0]
    a = S.feature_rows(cfg, torch.arange(100, 200))
    b = S.feature_rows(cfg, torch.tensor([150, 101, 199]))
    assert torch.equal(a[[50, 1, 99]], b)
    x = S.feature_rows(cfg, torch.arange(0, 20000)).double()
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1) < 0.01
