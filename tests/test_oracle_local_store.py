"""Pins for the CPU oracle's VIP-ordered local storage (Sec. 3.2, paragraph on host-to-device
transfer reduction; Sec. 4.1; Sec. 5, local partition storage on CPU versus GPU)."""
import itertools

import numpy as np
import torch

import oracle
from workloads import synth as S


def _scores(tiny):
    cfg, g, T, Tk = tiny
    pt, _ = oracle.vip(g.rowptr.numpy(), g.col.numpy(), Tk.numpy(), cfg.B, cfg.fanouts)
    return pt.astype(np.float32)


def test_capacity_is_floor_beta_n():
    assert oracle.local_capacity(0.10, 2500) == 250
    assert oracle.local_capacity(0.10, 7) == 0            # floor(0.7)
    assert oracle.local_capacity(0.5, 7) == 3
    assert oracle.local_capacity(1.0, 7) == 7
    assert oracle.local_capacity(0.0, 7) == 0
    assert oracle.local_capacity(2.0, 7) == 7             # never more than there is


def test_order_against_library_sort(tiny):
    cfg, g, T, Tk = tiny
    score = _scores(tiny)
    lo, hi = cfg.bounds()
    rank, order = oracle.local_rank(score, lo, hi)
    idx = np.arange(hi - lo)
    want = np.lexsort((idx, -score[lo:hi].astype(np.float64)))      # score desc, id asc
    assert np.array_equal(order, want)
    assert np.array_equal(rank[order], idx)                         # inverse permutations
    assert np.array_equal(np.sort(rank), idx)
    s = score[lo:hi][order]
    assert np.all(s[:-1] >= s[1:])


def test_order_in_a_partition_that_does_not_start_at_zero():
    rng = np.random.default_rng(5)
    score = rng.random(60).astype(np.float32)
    lo, hi = 20, 45
    rank, order = oracle.local_rank(score, lo, hi)
    want = np.lexsort((np.arange(25), -score[20:45].astype(np.float64)))
    assert np.array_equal(order, want)
    # scores outside [lo, hi) play no part
    score2 = score.copy()
    score2[:20] = 9.0
    score2[45:] = 9.0
    assert np.array_equal(oracle.local_rank(score2, lo, hi)[1], order)


def test_ties_zero_negative_and_nan_scores():
    score = np.array([0.5, 0.0, 0.5, -1.0, np.nan, 0.25, 0.0], dtype=np.float32)
    rank, order = oracle.local_rank(score, 0, 7)
    # 0.5 (ids 0, 2), 0.25 (id 5), then everything that counts as 0 in id order
    assert order.tolist() == [0, 2, 5, 1, 3, 4, 6]
    assert rank.tolist() == [0, 3, 1, 4, 5, 2, 6]
    # a constant score is the id order: the "no reorder" baseline
    r, o = oracle.local_rank(np.full(9, 0.3, np.float32), 2, 8)
    assert o.tolist() == list(range(6)) and r.tolist() == list(range(6))


def test_prefix_minimises_expected_host_reads_by_brute_force():
    """Keeping the first c of the order on the device leaves the smallest total score (expected
    number of host reads per minibatch) outside, over all subsets of size c (Sec. 3.2)."""
    rng = np.random.default_rng(11)
    score = rng.random(9).astype(np.float32)
    score[[2, 6]] = 0.0
    _, order = oracle.local_rank(score, 0, 9)
    s64 = score.astype(np.float64)
    for c in range(10):
        kept = s64[order[:c]].sum()
        best = max(s64[list(sub)].sum() for sub in itertools.combinations(range(9), c))
        assert abs(kept - best) < 1e-12


def test_split_gather_rows_tags_and_counts(tiny):
    cfg, g, T, Tk = tiny
    lo, hi = cfg.bounds()
    score = _scores(tiny)
    cache_ids = oracle.cache_select(score, lo, hi, cfg.K, cfg.alpha)
    local = S.feature_block(cfg, lo, hi).numpy()
    remote = S.feature_rows(cfg, S.remote_ids(cfg, 0, cfg.N - (hi - lo))).numpy()
    cache_rows = S.feature_rows(cfg, torch.from_numpy(cache_ids)).numpy()
    seeds = S.epoch_batches(cfg, Tk, 0)[0].numpy()
    m = oracle.sample_mfg(g.rowptr.numpy(), g.col.numpy(), seeds, cfg.fanouts, cfg.seed_sampler, 0)
    want = S.feature_rows(cfg, torch.from_numpy(m.node_ids)).numpy()
    rank, order = oracle.local_rank(score, lo, hi)
    is_local = (m.node_ids >= lo) & (m.node_ids < hi)
    is_cached = np.isin(m.node_ids, cache_ids)
    base_out, _, base_counts = oracle.gather(g.N, lo, hi, local, cache_rows, cache_ids, remote, m.node_ids)
    prev_host = None
    for beta in (0.0, 0.05, 0.3, 1.0):
        n_dev = oracle.local_capacity(beta, hi - lo)
        dev = local[order[:n_dev]]                       # device prefix: rows in rank order
        out, tag, counts = oracle.gather_split(g.N, lo, hi, dev, local, rank, n_dev, cache_rows, cache_ids,
                                               remote, m.node_ids)
        # the split never changes a byte of the result
        assert np.array_equal(out.view(np.uint32), want.view(np.uint32))
        assert np.array_equal(out.view(np.uint32), base_out.view(np.uint32))
        on_dev = np.zeros(m.node_ids.size, bool)
        on_dev[is_local] = rank[m.node_ids[is_local] - lo] < n_dev
        assert np.array_equal(tag == 0, on_dev)
        assert np.array_equal(tag == 3, is_local & ~on_dev)
        assert np.array_equal(tag == 1, is_cached)
        assert counts == (int(on_dev.sum()), int(is_cached.sum()), int((~is_local & ~is_cached).sum()),
                          int((is_local & ~on_dev).sum()))
        assert counts[0] + counts[3] == base_counts[0] and counts[1:3] == base_counts[1:3]
        if prev_host is not None:
            assert counts[3] <= prev_host                # a larger prefix never reads more from the host
        prev_host = counts[3]
    assert prev_host == 0                                # beta = 1: everything local is on the device
    # the device prefix is indexed by rank: a prefix laid out in id order must give wrong rows
    n_dev = oracle.local_capacity(0.3, hi - lo)
    wrong = local[:n_dev]
    out_w, tag_w, _ = oracle.gather_split(g.N, lo, hi, wrong, local, rank, n_dev, cache_rows, cache_ids, remote,
                                          m.node_ids)
    assert np.any(out_w[tag_w == 0] != want[tag_w == 0])
    # host rows are indexed by id: poisoning the host copy changes exactly the rows tagged 3
    bad = local + 1.0
    out_b, tag_b, _ = oracle.gather_split(g.N, lo, hi, local[order[:n_dev]], bad, rank, n_dev, cache_rows, cache_ids,
                                          remote, m.node_ids)
    assert np.array_equal(np.any(out_b != want, axis=1), tag_b == 3)


def test_vip_order_needs_a_smaller_prefix_than_id_order(tiny):
    """The effect the experiment on local storage reports: with the VIP order a small device prefix
    already serves a large share of the local reads, with the id order the served share grows about
    linearly; no order can beat the one made from the realised read counts."""
    cfg, g, T, Tk = tiny
    lo, hi = cfg.bounds()
    B, fanouts = 64, (5, 5)                              # small minibatches: access frequencies differ widely
    rowptr, col = g.rowptr.numpy(), g.col.numpy()
    pt, _ = oracle.vip(rowptr, col, Tk.numpy(), B, fanouts)
    score = pt.astype(np.float32)
    rank_vip, _ = oracle.local_rank(score, lo, hi)
    rank_id, _ = oracle.local_rank(np.zeros_like(score), lo, hi)
    reads = np.zeros(hi - lo)
    perm = np.random.default_rng(3).permutation(Tk.numpy())
    for b in range(0, perm.size - B + 1, B):
        m = oracle.sample_mfg(rowptr, col, perm[b:b + B], fanouts, 7, b // B)
        loc = m.node_ids[(m.node_ids >= lo) & (m.node_ids < hi)] - lo
        reads += np.bincount(loc, minlength=hi - lo)
    n_dev = oracle.local_capacity(0.2, hi - lo)
    served_vip = reads[rank_vip < n_dev].sum() / reads.sum()
    served_id = reads[rank_id < n_dev].sum() / reads.sum()
    served_best = np.sort(reads)[::-1][:n_dev].sum() / reads.sum()
    assert abs(served_id - 0.2) < 0.05
    assert served_vip > 2 * served_id
    assert served_vip <= served_best + 1e-12
    assert served_vip > 0.75 * served_best
