"""Pins for the CPU oracle's vertex-inclusion probabilities (Proposition 1, Sec. 3.1).

None of these re-types the oracle's loop: they check it against values worked by hand,
closed forms, inequalities that any correct evaluation satisfies, library routines in the
special cases the paper names (linear small-probability limit, full expansion), an exact
enumeration of the random process on graphs of <= 8 vertices, and a Monte-Carlo simulation.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def csr_from_adj(adj, N=None):
    N = N if N is not None else len(adj)
    rowptr = np.zeros(N + 1, dtype=np.int64)
    col = []
    for v in range(N):
        row = sorted(adj.get(v, [])) if isinstance(adj, dict) else sorted(adj[v])
        col.extend(row)
        rowptr[v + 1] = len(col)
    return rowptr, np.asarray(col, dtype=np.int32)


def golden_cases():
    out = {}
    for line in open(os.path.join(GOLD, "vip_closed_forms.txt")):
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        out[(parts[0], parts[1])] = np.array([float(x) for x in parts[2:]])
    return out


def test_hand_worked_cases():
    g = golden_cases()
    # A: out-star, also pins p^[0] = B/|T| = 1 and the direction (centre samples leaves)
    rp, col = csr_from_adj({0: [1, 2, 3, 4]}, 5)
    _, ph = oracle.vip(rp, col, [0], 1, [2])
    np.testing.assert_allclose(ph[0], g[("A", "p1")], rtol=0, atol=1e-15)
    # B: three training vertices pointing at one vertex
    rp, col = csr_from_adj({0: [3], 1: [3], 2: [3]}, 4)
    _, ph = oracle.vip(rp, col, [0, 1, 2], 1, [1])
    np.testing.assert_allclose(ph[0][3], g[("B", "p1_3")][0], rtol=1e-15)
    assert np.all(ph[0][:3] == 0)
    # C: directed path
    rp, col = csr_from_adj({0: [1], 1: [2], 2: [3]}, 4)
    pt, ph = oracle.vip(rp, col, [0], 1, [1, 1, 1])
    assert ph.tolist() == [[0, 1, 0, 0], [0, 0, 1, 0], [0, 0, 0, 1]]
    np.testing.assert_array_equal(pt, g[("C", "total")])
    # D: two hops, a product of two factors, and the product over hops in eq. (1)
    rp, col = csr_from_adj({0: [2, 3], 1: [3, 4, 5], 3: [5, 6]}, 7)
    pt, ph = oracle.vip(rp, col, [0, 1], 1, [1, 1])
    np.testing.assert_allclose(pt, g[("D", "total")], rtol=1e-14, atol=0)


def test_p0_and_clamp_and_hop0_flag():
    # m training vertices of out-degree dd all pointing at the same dd vertices
    m, dd, f, B = 7, 4, 2, 3
    adj = {v: list(range(m, m + dd)) for v in range(m)}
    rp, col = csr_from_adj(adj, m + dd)
    _, ph = oracle.vip(rp, col, list(range(m)), B, [f])
    want = 1 - (1 - (B / m) * min(1, f / dd)) ** m
    np.testing.assert_allclose(ph[0][m:], want, rtol=1e-14)
    # B > |T| clamps p^[0] to 1
    _, ph = oracle.vip(rp, col, list(range(m)), 100, [f])
    np.testing.assert_allclose(ph[0][m:], 1 - (1 - f / dd) ** m, rtol=1e-14)
    # eq. (1) as printed leaves hop 0 out; the flag multiplies (1 - p^[0]) in
    pt, _ = oracle.vip(rp, col, list(range(m)), B, [f])
    pt0, _ = oracle.vip(rp, col, list(range(m)), B, [f], include_hop0=True)
    assert np.all(pt[:m] == 0)
    np.testing.assert_allclose(pt0[:m], B / m, rtol=1e-14)
    np.testing.assert_allclose(pt0[m:], pt[m:], rtol=1e-14)


def test_x_equal_one_gives_exact_one():
    rp, col = csr_from_adj({0: [1, 2]}, 3)
    pt, ph = oracle.vip(rp, col, [0], 5, [2])
    assert ph[0].tolist() == [0.0, 1.0, 1.0] and pt.tolist() == [0.0, 1.0, 1.0]


def _transition(rp, col, f):
    """W[u, v] = min(1, f/d(v)) if u in adj(v): scipy sparse, built from the CSR transposed."""
    N = rp.size - 1
    d = np.diff(rp)
    src = np.repeat(np.arange(N), d)
    t = np.minimum(1.0, f / np.maximum(d, 1))
    return sp.csr_matrix((t[src], (col, src)), shape=(N, N))


def test_invariants_on_tiny(tiny):
    cfg, g, T, Tk = tiny
    rp, col = g.rowptr.numpy(), g.col.numpy()
    N = g.N
    for Tset, B in ((Tk.numpy(), cfg.B), (T.numpy(), cfg.B)):   # clamped and unclamped p^[0]
        pt, ph = oracle.vip(rp, col, Tset, B, cfg.fanouts)
        assert np.all((ph >= 0) & (ph <= 1)) and np.all((pt >= 0) & (pt <= 1))
        # support: p^[h](u) > 0 iff a walk of exactly h steps from T reaches u
        A = sp.csr_matrix((np.ones(col.size), col, rp), shape=(N, N))   # A[v,u]=1 iff u in adj(v)
        front = np.zeros(N, bool)
        front[Tset] = True
        reach = np.zeros(N, bool)
        for h in range(cfg.L):
            front = (A.T @ front.astype(np.float64)) > 0
            assert np.array_equal(ph[h] > 0, front)
            reach |= front
        assert np.array_equal(pt > 0, reach)
        # bounds per hop from the previous hop's vector
        prev = np.zeros(N)
        prev[Tset] = min(1.0, B / Tset.size)
        for h in range(cfg.L):
            W = _transition(rp, col, cfg.fanouts[h])
            X = W.multiply(prev[None, :]).tocsr()        # X[u,v] = x_h(v) on the edges into u
            s = np.asarray(X.sum(axis=1)).ravel()
            mx = np.asarray(X.max(axis=1).todense()).ravel()
            assert np.all(ph[h] >= mx - 1e-15)
            assert np.all(ph[h] <= np.minimum(1.0, s) + 1e-15)
            assert np.all(ph[h] >= s - 0.5 * s * s - 1e-15)
            prev = ph[h]


def test_literal_product_agrees_with_log_form(tiny):
    cfg, g, T, Tk = tiny
    rp, col = g.rowptr.numpy(), g.col.numpy()
    a_t, a_h = oracle.vip(rp, col, T.numpy(), cfg.B, cfg.fanouts)
    b_t, b_h = oracle.vip(rp, col, T.numpy(), cfg.B, cfg.fanouts, literal_product=True)
    np.testing.assert_allclose(a_h, b_h, rtol=1e-9, atol=1e-15)
    np.testing.assert_allclose(a_t, b_t, rtol=1e-9, atol=1e-15)


def test_monotone_in_fanout_and_batch(tiny):
    cfg, g, T, Tk = tiny
    rp, col = g.rowptr.numpy(), g.col.numpy()
    Tn = T.numpy()
    seq = [oracle.vip(rp, col, Tn, 64, f)[0] for f in ((5, 5, 5), (15, 10, 5), (20, 20, 20))]
    assert np.all(seq[0] <= seq[1] + 1e-15) and np.all(seq[1] <= seq[2] + 1e-15)
    assert np.any(seq[0] < seq[2])
    b = [oracle.vip(rp, col, Tn, B, cfg.fanouts)[0] for B in (16, 64, 256)]
    assert np.all(b[0] <= b[1] + 1e-15) and np.all(b[1] <= b[2] + 1e-15)


def test_small_probability_limit_is_a_sparse_matvec(tiny):
    """As B/|T| -> 0 the model is linear (the random-walk end of the continuum, Sec. 3.1)."""
    cfg, g, T, Tk = tiny
    rp, col = g.rowptr.numpy(), g.col.numpy()
    Tn = T.numpy()
    # make p^[0] tiny by a huge virtual training set: use B = 1 and scale afterwards
    pt, ph = oracle.vip(rp, col, Tn, 1, cfg.fanouts)       # p0 = 1e-3
    p = np.zeros(g.N)
    p[Tn] = 1.0 / Tn.size
    for h in range(cfg.L):
        p = _transition(rp, col, cfg.fanouts[h]) @ p
        nz = p > 0
        rel = np.abs(ph[h][nz] - p[nz]) / p[nz]
        assert rel.max() <= 2.0 * p.max() + 1e-12       # 1-prod(1-x) = sum x (1 + O(sum x))
        assert np.all(ph[h] <= p + 1e-18)


def test_full_expansion_is_boolean_frontier(tiny):
    """Fanouts above the largest degree and B = |T|: every x is 0 or 1 (Sec. 3.1)."""
    cfg, g, T, Tk = tiny
    rp, col = g.rowptr.numpy(), g.col.numpy()
    Tn = Tk.numpy()
    big = int(np.diff(rp).max()) + 1
    pt, ph = oracle.vip(rp, col, Tn, Tn.size, [big, big])
    A = sp.csr_matrix((np.ones(col.size), col, rp), shape=(g.N, g.N))
    front = np.zeros(g.N)
    front[Tn] = 1
    for h in range(2):
        front = ((A.T @ front) > 0).astype(np.float64)
        assert np.array_equal(ph[h], front)


# ----------------------------------------------------------------------------------------------
# exact enumeration of the random process of Sec. 3.1 on tiny graphs
# ----------------------------------------------------------------------------------------------

def enumerate_process(adj, N, T, p0, fanouts, batch_mode="bernoulli", B=None):
    """Exact distribution of the idealised process: start set -> union of sampled subsets -> ...

    Returns (p_hop[L][N], p_total[N]) as Fractions.  State = (frontier mask, seen-at-hops>=1 mask).
    """
    start = {}
    if batch_mode == "bernoulli":
        for bits in itertools.product([0, 1], repeat=len(T)):
            pr = Fraction(1)
            m = 0
            for b, v in zip(bits, T):
                pr *= p0 if b else (1 - p0)
                m |= b << v
            start[m] = start.get(m, 0) + pr
    else:
        combos = list(itertools.combinations(T, B))
        for c in combos:
            m = 0
            for v in c:
                m |= 1 << v
            start[m] = start.get(m, 0) + Fraction(1, len(combos))
    states = {(m, 0): pr for m, pr in start.items()}
    p_hop = []
    for f in fanouts:
        nxt = {}
        for (front, seen), pr in states.items():
            unions = {0: Fraction(1)}
            for v in range(N):
                if not (front >> v) & 1:
                    continue
                row = adj.get(v, [])
                c = min(f, len(row))
                if c == 0:
                    continue
                subs = list(itertools.combinations(row, c))
                w = Fraction(1, len(subs))
                new = {}
                for m, q in unions.items():
                    for s in subs:
                        mm = m
                        for u in s:
                            mm |= 1 << u
                        new[mm] = new.get(mm, 0) + q * w
                unions = new
            for m, q in unions.items():
                key = (m, seen | m)
                nxt[key] = nxt.get(key, 0) + pr * q
        states = nxt
        ph = [sum((pr for (m, _), pr in states.items() if (m >> u) & 1), Fraction(0)) for u in range(N)]
        p_hop.append(ph)
    p_tot = [sum((pr for (_, s), pr in states.items() if (s >> u) & 1), Fraction(0)) for u in range(N)]
    return p_hop, p_tot


def test_exact_enumeration_where_independence_holds():
    """Prop. 1 equals the exact process when batch membership is independent per training vertex
    and the walks into every vertex come from disjoint sets of roots (the proof's independence)."""
    adj = {0: [3, 5], 1: [4], 2: [4], 3: [7], 4: [5, 7], 5: [6]}
    N, T = 8, [0, 1, 2]
    rp, col = csr_from_adj(adj, N)
    for B, fan in ((1, (1, 1)), (2, (1, 2)), (1, (2, 1, 1)), (2, (1, 1, 1))):
        p0 = Fraction(B, len(T))
        eh, et = enumerate_process(adj, N, T, p0, fan)
        pt, ph = oracle.vip(rp, col, T, B, fan)
        for h in range(len(fan)):
            np.testing.assert_allclose(ph[h], [float(x) for x in eh[h]], rtol=1e-12, atol=1e-15)
        # eq. (1) multiplies over hops: exact here because a vertex reached at two different hops
        # (5 and 6) is reached through disjoint roots and through draws of different hops
        for u in range(N):
            assert abs(pt[u] - float(et[u])) <= 1e-12, (B, fan, u, pt[u], float(et[u]))


def test_exact_enumeration_gap_with_fixed_size_batches():
    """With B of |T| drawn without replacement and shared ancestors the formula is the paper's
    approximation; this records the size of the gap on small random graphs (not an equality)."""
    rng = np.random.default_rng(7)
    worst = 0.0
    for trial in range(6):
        N = 7
        adj = {}
        for v in range(N):
            k = int(rng.integers(0, 4))
            row = sorted(set(int(x) for x in rng.choice([u for u in range(N) if u != v], size=k, replace=False)))
            if row:
                adj[v] = row
        T = [0, 1, 2]
        rp, col = csr_from_adj(adj, N)
        eh, et = enumerate_process(adj, N, T, None, (2, 1), batch_mode="fixed", B=2)
        pt, ph = oracle.vip(rp, col, T, 2, (2, 1))
        # hop 1 with a fixed-size batch: membership is negatively associated, so the exact value
        # is >= the formula; and the formula is exact where a single training vertex points at u
        e1 = np.array([float(x) for x in eh[0]])
        assert np.all(e1 >= ph[0] - 1e-12)
        indeg_from_T = np.zeros(N, int)
        for v in T:
            for u in adj.get(v, []):
                indeg_from_T[u] += 1
        single = indeg_from_T == 1
        np.testing.assert_allclose(ph[0][single], e1[single], rtol=1e-12)
        worst = max(worst, float(np.max(np.abs(pt - np.array([float(x) for x in et])))))
    assert worst < 0.25       # a loose sanity bound; the gap is the model's, not the code's


# ----------------------------------------------------------------------------------------------
# Monte-Carlo simulation of the idealised process (independent of the oracle's sampler)
# ----------------------------------------------------------------------------------------------

def test_monte_carlo_on_a_forest():
    """On a forest (one in-neighbour per vertex) with Bernoulli batches Prop. 1 is exact; a
    numpy simulation of the process must agree within binomial error."""
    rng = np.random.default_rng(11)
    N, roots = 300, 12
    parent = np.full(N, -1)
    adj = {}
    for u in range(roots, N):
        p = int(rng.integers(0, u))
        parent[u] = p
        adj.setdefault(p, []).append(u)
    rp, col = csr_from_adj(adj, N)
    T = list(range(roots))
    B, fan = 4, (2, 1, 2)
    pt, ph = oracle.vip(rp, col, T, B, fan)
    trials = 20000
    cnt_h = np.zeros((len(fan), N))
    cnt_t = np.zeros(N)
    p0 = B / len(T)
    for _ in range(trials):
        front = [v for v in T if rng.random() < p0]
        seen = set()
        for h, f in enumerate(fan):
            nxt = set()
            for v in front:
                row = adj.get(v, [])
                if not row:
                    continue
                c = min(f, len(row))
                nxt.update(rng.choice(row, size=c, replace=False).tolist())
            for u in nxt:
                cnt_h[h, u] += 1
            seen |= nxt
            front = list(nxt)
        for u in seen:
            cnt_t[u] += 1
    for est, p in ((cnt_h[h] / trials, ph[h]) for h in range(len(fan))):
        sigma = np.sqrt(np.maximum(p * (1 - p), 1e-9) / trials)
        assert np.all(np.abs(est - p) <= 5 * sigma + 1e-4)
    # in a forest each vertex is reachable at one hop only, so eq. (1) is exact as well
    sigma = np.sqrt(np.maximum(pt * (1 - pt), 1e-9) / trials)
    assert np.all(np.abs(cnt_t / trials - pt) <= 5 * sigma + 1e-4)


def test_direction_is_not_transposed():
    """adj(v) is what v samples from: probability flows from v to the members of its row only."""
    rp, col = csr_from_adj({0: [1], 2: [0]}, 3)       # 0 samples 1; 2 samples 0
    pt, ph = oracle.vip(rp, col, [0], 1, [1, 1])
    assert ph[0].tolist() == [0.0, 1.0, 0.0]           # 2 is never reached from 0
    assert pt.tolist() == [0.0, 1.0, 0.0]


def test_fanout_order_hop1_uses_first_entry():
    rp, col = csr_from_adj({0: [1, 2, 3, 4], 1: [5, 6]}, 7)
    _, ph = oracle.vip(rp, col, [0], 1, [2, 1])
    np.testing.assert_allclose(ph[0][1:5], 0.5)          # f_1 = 2 over d = 4
    np.testing.assert_allclose(ph[1][5:7], 0.5 * 0.5)    # f_2 = 1 over d = 2
    _, ph = oracle.vip(rp, col, [0], 1, [1, 2])
    np.testing.assert_allclose(ph[0][1:5], 0.25)
    np.testing.assert_allclose(ph[1][5:7], 0.25 * 1.0)
