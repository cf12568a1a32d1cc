"""Pins for the CPU oracle's general form of Proposition 1 (arbitrary initial and transition
probabilities, Sec. 3.1) and for the independent-inclusion sampler that realises given
transition probabilities exactly."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from workloads import synth as S


def csr_from_adj(adj, N):
    rp = np.zeros(N + 1, dtype=np.int64)
    col = []
    for v in range(N):
        row = adj.get(v, [])
        col.extend(row)
        rp[v + 1] = rp[v] + len(row)
    return rp, np.array(col, dtype=np.int32)


def _uniform_t(rp, f):
    d = np.diff(rp)
    per_row = np.minimum(1.0, f / np.maximum(d, 1)).astype(np.float32)
    return np.repeat(per_row, d)


# ----------------------------------------------------------------------------------------------
# general VIP
# ----------------------------------------------------------------------------------------------

def test_uniform_instantiation_reduces_to_the_pinned_uniform_oracle(tiny):
    """t = min(1, f_h/d(v)) and p0 = min(1, B/|T|) on T is the instantiation of Sec. 3.1."""
    cfg, g, T, Tk = tiny
    rp, col = g.rowptr.numpy(), g.col.numpy()
    for B, fan in ((cfg.B, cfg.fanouts), (16, (3, 2)), (1, (1,))):
        p0 = np.zeros(g.N, dtype=np.float32)
        p0[Tk.numpy()] = min(1.0, B / Tk.numel())
        # the general oracle takes float32 probabilities, the uniform one B and f: the inputs differ by
        # float32 rounding (6e-8 each), hence the tolerance
        t = [_uniform_t(rp, f) for f in fan]
        pt, ph = oracle.vip_general(rp, col, p0, t, len(fan))
        rt, rh = oracle.vip(rp, col, Tk.numpy(), B, fan)
        np.testing.assert_allclose(ph, rh, rtol=5e-7, atol=1e-300)
        np.testing.assert_allclose(pt, rt, rtol=5e-7, atol=1e-300)
        assert np.array_equal(pt == 0, rt == 0)
    # with probabilities that float32 holds exactly the two oracles agree to rounding order
    adj = {0: [1, 2, 3, 4], 1: [2, 5], 2: [5, 6, 7, 3], 3: [7]}
    rp, col = csr_from_adj(adj, 8)
    p0 = np.zeros(8, np.float32)
    p0[[0, 1]] = 0.5                                      # B = 1, |T| = 2
    pt, ph = oracle.vip_general(rp, col, p0, [_uniform_t(rp, 2), _uniform_t(rp, 1)], 2)
    rt, rh = oracle.vip(rp, col, [0, 1], 1, (2, 1))
    np.testing.assert_allclose(ph, rh, rtol=1e-14)
    np.testing.assert_allclose(pt, rt, rtol=1e-14)


def test_hand_worked_two_hops():
    # 0 -> {1 (t=.5), 2 (t=.25)}, 1 -> {2 (t=.5)}; p0 = (.5, .25, 0)
    rp, col = csr_from_adj({0: [1, 2], 1: [2]}, 3)
    t = np.array([0.5, 0.25, 0.5], dtype=np.float32)
    p0 = np.array([0.5, 0.25, 0.0], dtype=np.float32)
    pt, ph = oracle.vip_general(rp, col, p0, t, 2)
    h1 = [0.0, 0.25, 1 - (1 - 0.125) * (1 - 0.125)]
    h2 = [0.0, 0.0, 0.5 * 0.25]
    np.testing.assert_allclose(ph[0], h1, rtol=1e-15)
    np.testing.assert_allclose(ph[1], h2, rtol=1e-15)
    np.testing.assert_allclose(pt, [0.0, 0.25, 1 - (1 - h1[2]) * (1 - h2[2])], rtol=1e-15)
    # hop 0 multiplied in
    pt0, _ = oracle.vip_general(rp, col, p0, t, 2, include_hop0=True)
    np.testing.assert_allclose(pt0, [0.5, 1 - 0.75 * 0.75, pt[2]], rtol=1e-15)
    # per-hop matrices: hop 2 with its own probabilities
    t2 = np.array([0.0, 0.0, 1.0], dtype=np.float32)
    _, ph2 = oracle.vip_general(rp, col, p0, [t, t2], 2)
    np.testing.assert_allclose(ph2[1], [0.0, 0.0, 0.25], rtol=1e-15)


def test_values_outside_the_unit_interval_are_refused():
    rp, col = csr_from_adj({0: [1]}, 2)
    ok_p, ok_t = np.array([0.5, 0], np.float32), np.array([0.5], np.float32)
    for bad in (1.5, -0.1, np.nan):
        with pytest.raises(ValueError):
            oracle.vip_general(rp, col, np.array([bad, 0], np.float32), ok_t, 1)
        with pytest.raises(ValueError):
            oracle.vip_general(rp, col, ok_p, np.array([bad], np.float32), 1)


def test_small_probability_limit_is_a_sparse_matvec(tiny):
    """For tiny probabilities the products linearise: p^[h] = A_h^T p^[h-1] with A_h[v, u] = t_h(u, v)."""
    cfg, g, T, Tk = tiny
    rp, col = g.rowptr.numpy(), g.col.numpy()
    rng = np.random.default_rng(3)
    t = [rng.random(col.size).astype(np.float32) for _ in range(2)]
    p0 = (rng.random(g.N) * 1e-9).astype(np.float32)
    _, ph = oracle.vip_general(rp, col, p0, t, 2)
    A = [sp.csr_matrix((a.astype(np.float64), col, rp), shape=(g.N, g.N)) for a in t]
    l1 = A[0].T @ p0.astype(np.float64)
    l2 = A[1].T @ l1
    np.testing.assert_allclose(ph[0], l1, rtol=1e-6, atol=1e-300)
    np.testing.assert_allclose(ph[1], l2, rtol=1e-6, atol=1e-300)


def test_direction_and_alignment_of_the_edge_probabilities():
    # t is aligned with col: the probability sits on the edge (row vertex samples col entry), not on its reverse
    rp, col = csr_from_adj({0: [1, 2], 2: [0]}, 3)
    p0 = np.array([1.0, 0.0, 0.0], np.float32)
    t = np.array([0.25, 0.75, 0.5], np.float32)
    _, ph = oracle.vip_general(rp, col, p0, t, 1)
    np.testing.assert_allclose(ph[0], [0.0, 0.25, 0.75], rtol=1e-15)


def _enumerate_independent(adj_t, N, p0, L):
    """Exact hop-wise inclusion probabilities of the process with independent batch membership and
    independent inclusion of every (hop, edge), by enumeration with exact fractions."""
    states = {}
    for members in itertools.product([0, 1], repeat=N):
        pr = Fraction(1)
        m = 0
        for v, b in enumerate(members):
            pr *= p0[v] if b else 1 - p0[v]
            m |= b << v
        if pr:
            states[(m, 0)] = states.get((m, 0), 0) + pr
    p_hop = []
    for h in range(L):
        nxt = {}
        for (front, seen), pr in states.items():
            edges = [(v, u, tt) for v in range(N) if (front >> v) & 1 for (u, tt) in adj_t[h].get(v, [])]
            unions = {0: Fraction(1)}
            for (_, u, tt) in edges:
                new = {}
                for m, q in unions.items():
                    if tt:
                        new[m | (1 << u)] = new.get(m | (1 << u), 0) + q * tt
                    if tt != 1:
                        new[m] = new.get(m, 0) + q * (1 - tt)
                unions = new
            for m, q in unions.items():
                key = (m, seen | m)
                nxt[key] = nxt.get(key, 0) + pr * q
        states = nxt
        p_hop.append([sum((pr for (m, _), pr in states.items() if (m >> u) & 1), Fraction(0)) for u in range(N)])
    p_tot = [sum((pr for (_, s), pr in states.items() if (s >> u) & 1), Fraction(0)) for u in range(N)]
    return p_hop, p_tot


def test_exact_enumeration_where_independence_holds():
    """On an in-tree (every vertex samples at most one neighbour, so the ancestries of a vertex's
    in-neighbours are disjoint) with independent batch membership, Prop. 1 is exact for arbitrary
    dyadic p0 and t, hop by hop and in total."""
    # edges point towards the root 6: 0->4, 1->4, 2->5, 3->5, 4->6, 5->6
    out = {0: 4, 1: 4, 2: 5, 3: 5, 4: 6, 5: 6}
    N, L = 7, 2
    tq = [{0: Fraction(1, 2), 1: Fraction(3, 4), 2: Fraction(1, 4), 3: Fraction(1), 4: Fraction(1, 2), 5: Fraction(1, 8)},
          {0: Fraction(1, 4), 1: Fraction(1, 2), 2: Fraction(1), 3: Fraction(1, 2), 4: Fraction(3, 4), 5: Fraction(1, 2)}]
    p0q = [Fraction(1, 2), Fraction(1, 4), Fraction(3, 4), Fraction(1, 2), Fraction(1, 4), Fraction(0), Fraction(1, 8)]
    adj = {v: [u] for v, u in out.items()}
    rp, col = csr_from_adj(adj, N)
    t = [np.array([float(tq[h][v]) for v in range(N) if v in out], dtype=np.float32) for h in range(L)]
    adj_t = [{v: [(u, tq[h][v])] for v, u in out.items()} for h in range(L)]
    eh, et = _enumerate_independent(adj_t, N, p0q, L)
    pt, ph = oracle.vip_general(rp, col, np.array([float(x) for x in p0q], np.float32), t, L)
    for h in range(L):
        np.testing.assert_allclose(ph[h], [float(x) for x in eh[h]], rtol=1e-13, atol=1e-300)
    np.testing.assert_allclose(pt, [float(x) for x in et], rtol=1e-13, atol=1e-300)


def test_gap_where_walks_share_ancestors_is_the_models():
    """A diamond (0 -> 1, 0 -> 2, 1 -> 3, 2 -> 3): the two ways into 3 share vertex 0, the formula
    treats them as independent.  Hop 1 stays exact; the hop-2 value is the product form, above the exact one."""
    adj = {0: [1, 2], 1: [3], 2: [3]}
    rp, col = csr_from_adj(adj, 4)
    half = Fraction(1, 2)
    adj_t = [{0: [(1, half), (2, half)], 1: [(3, half)], 2: [(3, half)]}] * 2
    p0q = [half, Fraction(0), Fraction(0), Fraction(0)]
    eh, _ = _enumerate_independent(adj_t, 4, p0q, 2)
    _, ph = oracle.vip_general(rp, col, np.array([0.5, 0, 0, 0], np.float32), np.full(4, 0.5, np.float32), 2)
    np.testing.assert_allclose(ph[0], [float(x) for x in eh[0]], rtol=1e-15)
    formula = 1 - (1 - 0.5 * 0.25) ** 2
    assert abs(ph[1][3] - formula) < 1e-15
    assert float(eh[1][3]) < formula and formula - float(eh[1][3]) < 0.02


# ----------------------------------------------------------------------------------------------
# independent-inclusion sampler
# ----------------------------------------------------------------------------------------------

def test_sampler_threshold_rule_and_layout_by_reference_loops(tiny):
    """Edge k of a target's row is taken iff rand32(seed, batch, hop, v, k) < floor(t * 2^32); the MFG
    is laid out like the fanout sampler's (checked with plain Python loops and np.unique)."""
    cfg, g, T, Tk = tiny
    rp, col = g.rowptr.numpy(), g.col.numpy()
    rng = np.random.default_rng(9)
    t = [rng.random(col.size).astype(np.float32) * 0.4 for _ in range(2)]
    t[0][rp[Tk.numpy()[0]]:rp[Tk.numpy()[0] + 1]] = 1.0            # one seed takes its whole row
    seeds = Tk.numpy()[:40]
    m = oracle.sample_mfg_general(rp, col, t, seeds, 2, 77, 5)
    S_prev = list(seeds)
    for h in (1, 2):
        flat, ptr = [], [0]
        for v in S_prev:
            for k in range(rp[v + 1] - rp[v]):
                e = rp[v] + k
                thr = int(float(t[h - 1][e]) * 4294967296.0)
                if oracle.rand32(77, 5, h, int(v), k) < thr:
                    flat.append(int(col[e]))
            ptr.append(len(flat))
        assert m.e[h] == len(flat) and m.indptr[h - 1].tolist() == ptr
        seen = set(S_prev)
        S_h = list(S_prev)
        for x in flat:
            if x not in seen:
                seen.add(x)
                S_h.append(x)
        assert m.n[h] == len(S_h)
        assert m.node_ids[:m.n[h]].tolist() == S_h
        index = {x: i for i, x in enumerate(S_h)}
        assert m.src[h - 1].tolist() == [index[x] for x in flat]
        S_prev = S_h
    # the seed with t = 1 took every neighbour, in row order
    v0 = int(seeds[0])
    row = col[rp[v0]:rp[v0 + 1]]
    got = m.node_ids[m.src[0][m.indptr[0][0]:m.indptr[0][1]]]
    assert np.array_equal(got, row)
    assert np.unique(m.node_ids).size == m.node_ids.size


def test_sampler_t_zero_and_t_one():
    adj = {0: [1, 2], 1: [3], 2: [3, 4], 3: [5]}
    rp, col = csr_from_adj(adj, 6)
    none = oracle.sample_mfg_general(rp, col, np.zeros(6, np.float32), [0], 3, 1, 0)
    assert none.n == [1, 1, 1, 1] and none.e == [0, 0, 0, 0]
    full = oracle.sample_mfg_general(rp, col, np.ones(6, np.float32), [0], 3, 1, 0)
    # full expansion: S_h = everything within h steps, all rows re-expanded every hop
    assert full.node_ids.tolist() == [0, 1, 2, 3, 4, 5]
    assert full.n == [1, 3, 5, 6] and full.e == [0, 2, 5, 6]


def test_realised_edge_frequencies_match_t():
    """Over many minibatches an edge of a seed's row is taken with probability t (binomial, 5 sigma)."""
    rng = np.random.default_rng(4)
    d = 12
    adj = {0: list(range(1, d + 1))}
    rp, col = csr_from_adj(adj, d + 1)
    t = rng.random(d).astype(np.float32)
    t[0], t[1] = 0.0, 1.0
    trials = 4000
    hits = np.zeros(d)
    for b in range(trials):
        m = oracle.sample_mfg_general(rp, col, t, [0], 1, 123, b)
        hits[m.node_ids[1:] - 1] += 1
    sd = np.sqrt(np.maximum(t * (1 - t), 1e-12) / trials)
    assert np.all(np.abs(hits / trials - t) <= 5 * sd + 1e-12)
    assert hits[0] == 0 and hits[1] == trials


def test_sampled_frequencies_match_general_vip_on_an_in_tree():
    """Monte Carlo with the sampler itself against the general formula, where the formula is exact:
    seeds drawn independently per vertex, in-tree, two hops.  The sampler re-expands all of S_{h-1}
    (an MFG needs the targets' own rows) while the model's hop-2 frontier is only what hop 1 sampled;
    here the seeds are leaves that nothing points at, so the model's hop-2 set is exactly the sources
    of the hop-2 edges whose target is not a seed."""
    rng = np.random.default_rng(21)
    N, leaves = 40, 24
    adj = {v: [int(rng.integers(max(v + 1, leaves), N))] for v in range(N - 1)}
    rp, col = csr_from_adj(adj, N)
    t = [rng.random(col.size).astype(np.float32) * 0.8 + 0.1 for _ in range(2)]
    p0 = np.zeros(N, np.float32)
    p0[:leaves] = 0.3
    _, ph = oracle.vip_general(rp, col, p0, t, 2)
    trials = 6000
    hop1, hop2 = np.zeros(N), np.zeros(N)
    for b in range(trials):
        seeds = np.flatnonzero(rng.random(N) < p0).astype(np.int32)
        m = oracle.sample_mfg_general(rp, col, t, seeds, 2, 5, b)
        if m.e[1]:
            hop1[np.unique(m.node_ids[m.src[0]])] += 1
        first = m.indptr[1][m.n[0]]                      # hop-2 edges of the targets after the seeds
        if m.e[2] > first:
            hop2[np.unique(m.node_ids[m.src[1][first:]])] += 1
    for got, want in ((hop1, ph[0]), (hop2, ph[1])):
        sd = np.sqrt(np.maximum(want * (1 - want), 1e-9) / trials)
        assert np.all(np.abs(got / trials - want) <= 5 * sd + 1e-9)
    assert hop2.sum() > 0
