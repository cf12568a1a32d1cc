"""GPU parity: the HIP path, called through the C interface, against the CPU oracle on the same
seeded inputs.  Integer outputs (MFGs, relabel maps, cache membership, gathered rows, counts) must
match bit for bit; fp32 vertex-inclusion probabilities within 1e-5 relative (floor 1e-37)."""
import numpy as np
import pytest
import torch

import oracle
from workloads import synth as S

pytestmark = pytest.mark.gpu

VIP_RTOL, VIP_FLOOR = 1e-5, 1e-37


def _say(*a):
    print("[case]", *a, flush=True)


@pytest.fixture(scope="module")
def spp():
    import paper_2305_03152_amd as m
    m.load_library()
    return m


# Every case runs twice: with the transposed edges in row blocks (graphs whose per-vertex vectors stay in
# the caches) and the sampler's hops deduplicated in LDS (what these sizes get by default), and with the
# forms that large inputs get, forced here at small sizes: the chunked layout of graphs above 2^23 vertices
# and the sampler's id table in global memory (hops of more than 131072 ids).
_CHUNKED = False


@pytest.fixture(scope="module", params=["row-blocks", "chunked"], autouse=True)
def layout(request):
    global _CHUNKED
    import functools
    import paper_2305_03152_amd as m
    _CHUNKED = request.param == "chunked"
    saved = (m.sample_mfg, m.sample_mfg_multi)
    if _CHUNKED:
        m.sample_mfg = functools.partial(saved[0], global_table=True)
        m.sample_mfg_multi = functools.partial(saved[1], global_table=True)
    yield request.param
    m.sample_mfg, m.sample_mfg_multi = saved
    _CHUNKED = False


@pytest.fixture(scope="module")
def ctx(spp, layout):
    c = spp.Context(0)
    yield c
    c.close()


class Case:
    """A workload on the GPU plus the same arrays on the host for the oracle."""

    def __init__(self, spp, ctx, cfg, gen_device="cpu", in_lists=True):
        self.cfg = cfg
        dev = torch.device("cuda:0")
        g = S.make_graph(cfg, gen_device)
        self.N, self.M = g.N, g.M
        self.rowptr_d, self.col_d = g.rowptr.to(dev), g.col.to(dev)
        self.rp, self.col = g.rowptr.cpu().numpy(), g.col.cpu().numpy()
        T = S.make_training_set(cfg, gen_device)
        self.Tk_d = S.local_training_set(cfg, T).to(dev)
        self.Tk = self.Tk_d.cpu().numpy()
        self.T_all = T.cpu().numpy()
        self.lo, self.hi = cfg.bounds()
        self.G = spp.Graph(ctx, self.rowptr_d, self.col_d, in_lists=in_lists, chunked=_CHUNKED)

    def features(self):
        cfg = self.cfg
        dev = torch.device("cuda:0")
        self.local_d = S.feature_block(cfg, self.lo, self.hi, dev)
        nrem = cfg.N - (self.hi - self.lo)
        self.remote = torch.empty((nrem, cfg.D), dtype=cfg.torch_dtype).pin_memory()
        for a in range(0, nrem, 1 << 20):
            b = min(nrem, a + (1 << 20))
            self.remote[a:b].copy_(S.feature_rows(cfg, S.remote_ids(cfg, a, b, dev)))
        torch.cuda.synchronize()


def _bits(a):
    a = np.ascontiguousarray(a)
    return a.view({2: np.uint16, 4: np.uint32}[a.dtype.itemsize])


def _np(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy()
    return t.cpu().numpy()


def _check_vip(p_gpu, p_ref):
    p = p_gpu.cpu().numpy().astype(np.float64)
    err = np.abs(p - p_ref)
    tol = VIP_RTOL * p_ref + VIP_FLOOR
    bad = np.flatnonzero(err > tol)
    assert bad.size == 0, (bad[:5], p[bad[:5]], p_ref[bad[:5]])
    assert np.all(p[p_ref == 0] == 0) and np.all(p_ref[p == 0] < 1e-37)


def _check_mfg(m, ref, L):
    assert m.n == ref.n and m.e == ref.e, (m.n, ref.n, m.e, ref.e)
    assert np.array_equal(m.node_ids[:m.n[L]].cpu().numpy(), ref.node_ids)
    for h in range(L):
        assert np.array_equal(m.indptr[h][:m.n[h] + 1].cpu().numpy(), ref.indptr[h]), f"indptr hop {h + 1}"
        assert np.array_equal(m.src[h][:m.e[h + 1]].cpu().numpy(), ref.src[h]), f"src hop {h + 1}"


# ----------------------------------------------------------------------------------------------
# tiny graphs with known answers first: a fault here names the kernel at once
# ----------------------------------------------------------------------------------------------

def _mini_graph(spp, ctx, adj, N):
    rp = np.zeros(N + 1, dtype=np.int64)
    col = []
    for v in range(N):
        col.extend(sorted(adj.get(v, [])))
        rp[v + 1] = len(col)
    col = np.asarray(col, dtype=np.int32)
    dev = torch.device("cuda:0")
    G = spp.Graph(ctx, torch.from_numpy(rp).to(dev), torch.from_numpy(col).to(dev) if col.size else torch.zeros(0, dtype=torch.int32, device=dev),
                  in_lists=True, chunked=_CHUNKED)
    return G, rp, col


def test_vip_hand_worked(spp, ctx):
    _say("vip hand-worked graphs")
    dev = torch.device("cuda:0")
    G, rp, col = _mini_graph(spp, ctx, {0: [2, 3], 1: [3, 4, 5], 3: [5, 6]}, 7)
    T = torch.tensor([0, 1], dtype=torch.int32, device=dev)
    p, ph = spp.vip_propagate(ctx, G, T, 1, (1, 1), per_hop=True)
    want = [0, 0, 0.25, 0.375, 1 / 6, 31 / 96, 3 / 16]
    np.testing.assert_allclose(p.cpu().numpy(), want, rtol=1e-6)
    ref_t, ref_h = oracle.vip(rp, col, [0, 1], 1, (1, 1))
    np.testing.assert_allclose(ph.cpu().numpy(), ref_h, rtol=1e-6)
    # x = 1 exactly gives p = 1 exactly; clamp of p^[0]; hop 0 included on request
    G2, rp2, col2 = _mini_graph(spp, ctx, {0: [1, 2]}, 3)
    T2 = torch.tensor([0], dtype=torch.int32, device=dev)
    assert spp.vip_propagate(ctx, G2, T2, 5, (2,)).cpu().tolist() == [0.0, 1.0, 1.0]
    p0 = spp.vip_propagate(ctx, G, T, 1, (1, 1), include_hop0=True)
    ref0, _ = oracle.vip(rp, col, [0, 1], 1, (1, 1), include_hop0=True)
    np.testing.assert_allclose(p0.cpu().numpy(), ref0, rtol=1e-6)
    # a graph without edges
    G3, _, _ = _mini_graph(spp, ctx, {}, 5)
    assert spp.vip_propagate(ctx, G3, T2, 1, (3, 3)).cpu().tolist() == [0.0] * 5


def test_sampler_mini(spp, ctx):
    _say("sampler on a 3-vertex graph, zero-degree vertex, empty batch")
    dev = torch.device("cuda:0")
    G, rp, col = _mini_graph(spp, ctx, {0: [1, 2], 2: [0]}, 3)
    for seeds, fan in (([1], (2, 2)), ([0, 1], (2,)), ([], (2,)), ([2, 0], (1, 1, 1))):
        s = torch.tensor(seeds, dtype=torch.int32, device=dev)
        m = spp.sample_mfg(ctx, G, s, fan, 1, 0)
        ref = oracle.sample_mfg(rp, col, seeds, fan, 1, 0)
        _check_mfg(m, ref, len(fan))


def _random_graph(rng, N, degrees):
    """CSR with the given out-degree per vertex, neighbours drawn without repetition, sorted."""
    rp = np.zeros(N + 1, dtype=np.int64)
    cols = []
    for v in range(N):
        d = int(degrees[v])
        cols.append(np.sort(rng.choice(N, size=d, replace=False)).astype(np.int32))
        rp[v + 1] = rp[v] + d
    return rp, (np.concatenate(cols) if cols else np.zeros(0, np.int32))


@pytest.mark.parametrize("fanouts", [(64,), (63, 2), (33, 3), (32, 2), (17, 9, 1), (16, 16), (9, 8, 7), (8, 1, 8), (1,) * 8,
                                     (2,) * 8, (3, 1, 2, 1, 3, 1, 2, 1)])
def test_sampler_and_vip_shape_sweep(spp, ctx, fanouts):
    """Every lane-group width of the sampler (8/16/32/64), the largest fanout and the largest number
    of hops, on a graph whose degrees sit at and around each fanout (0, 1, f-1, f, f+1, hubs);
    vertex-inclusion probabilities on the same graph."""
    rng = np.random.default_rng(sum(fanouts) * 131 + len(fanouts))
    N = 700
    marks = sorted({0, 1, 2, 600} | {max(0, f + d) for f in fanouts for d in (-1, 0, 1)})
    degrees = rng.choice(np.asarray(marks), size=N)
    degrees[:8] = [0, 1, 600, 65, 64, 63, 2, 0]
    rp, col = _random_graph(rng, N, degrees)
    dev = torch.device("cuda:0")
    G = spp.Graph(ctx, torch.from_numpy(rp).to(dev), torch.from_numpy(col).to(dev), in_lists=True, chunked=_CHUNKED)
    L = len(fanouts)
    seeds = np.concatenate([np.arange(8), 8 + rng.permutation(N - 8)[:43]]).astype(np.int32)    # distinct, as a minibatch is
    _say("shape sweep: fanouts", fanouts, "M", col.size)
    for bi in (0, 7):
        m = spp.sample_mfg(ctx, G, torch.from_numpy(seeds).to(dev), fanouts, 99, bi)
        _check_mfg(m, oracle.sample_mfg(rp, col, seeds, fanouts, 99, bi), L)
    items = [(torch.from_numpy(seeds[:k]).to(dev), 20 + k, spp.MFGBuffers("cuda", 64, fanouts, N)) for k in (51, 1, 17)]
    spp.sample_mfg_multi(ctx, G, items, fanouts, 5)
    for (sd, bi, m), k in zip(items, (51, 1, 17)):
        _check_mfg(m, oracle.sample_mfg(rp, col, seeds[:k], fanouts, 5, bi), L)
    T = np.sort(seeds)
    p, ph = spp.vip_propagate(ctx, G, torch.from_numpy(T).to(dev), 16, fanouts, per_hop=True)
    ref_t, ref_h = oracle.vip(rp, col, T, 16, fanouts)
    _check_vip(p, ref_t)
    for h in range(L):
        _check_vip(ph[h], ref_h[h])
    G.close()


def test_stream_rates_of_the_plain_kernels(spp, ctx, layout):
    """The streaming kernels behind the bench line's measured HBM rates: three positive rates, far above what a
    host link could move, and arguments that make no sense are refused."""
    if layout != "row-blocks":
        pytest.skip("once is enough")
    r = spp.stream_rates(ctx, 256 << 20, 3)
    _say("stream rates over 256 MiB:", r)
    assert set(r) == {"read_only", "copy_read_plus_write", "write_only"}
    assert all(v > 500.0 for v in r.values()), r
    with pytest.raises(spp.SppError):
        spp.stream_rates(ctx, 256 << 20, 0)


def test_sampler_hops_on_both_sides_of_the_lds_capacity(spp, ctx):
    """One call whose minibatches take different forms of the deduplication at their last hop: a few
    hundred ids (one LDS partition), just under 16 x 8192 ids (sixteen partitions, nearly full) and twice
    that (the table in global memory), decided per minibatch on the device."""
    rng = np.random.default_rng(4711)
    N, d = 400_000, 32
    t = np.sort(rng.integers(0, N, size=(N, d), dtype=np.int64), axis=1)
    keep = np.ones_like(t, dtype=bool)
    keep[:, 1:] = t[:, 1:] != t[:, :-1]                    # rows sort-uniqued
    rp = np.zeros(N + 1, dtype=np.int64)
    rp[1:] = np.cumsum(keep.sum(axis=1))
    col = t[keep].astype(np.int32)
    dev = torch.device("cuda:0")
    G = spp.Graph(ctx, torch.from_numpy(rp).to(dev), torch.from_numpy(col).to(dev))
    fanouts = (15, 10)
    perm = rng.permutation(N).astype(np.int32)
    sizes = (40, 690, 1500, 5)
    seeds = [np.ascontiguousarray(perm[1000 * k:1000 * k + n]) for k, n in enumerate(sizes)]
    items = [(torch.from_numpy(s_).to(dev), 300 + k, spp.MFGBuffers("cuda", 1500, fanouts, N)) for k, s_ in enumerate(seeds)]
    spp.sample_mfg_multi(ctx, G, items, fanouts, 31337)
    keys = []
    for (sd, bi, m), s_ in zip(items, seeds):
        ref = oracle.sample_mfg(rp, col, s_, fanouts, 31337, bi)
        _check_mfg(m, ref, 2)
        keys.append(ref.n[1] + ref.e[2])
    _say("ids at the last hop:", keys)
    if not _CHUNKED:                                       # (the other run of this module forces the global table everywhere)
        assert keys[0] < 8192 and 8 * 8192 < keys[1] <= 16 * 8192 < keys[2], keys
    G.close()


def test_vip_long_rows_in_the_frontier(spp, ctx):
    """Frontier rows of 4095 to 12000 entries: the push hops list such a row in pieces of 4096 entries
    that different workgroups walk (both entry points, with and without the row-block structure)."""
    rng = np.random.default_rng(77)
    N = 20000
    degrees = np.full(N, 28)         # M large enough for a hop-1 frontier of 34k out-edges to count as sparse
    hubs = {5: 12000, 300: 4096, 301: 4097, 7000: 4095, 19999: 9000}
    for v, d in hubs.items():
        degrees[v] = d
    rp = np.zeros(N + 1, dtype=np.int64)
    rp[1:] = np.cumsum(degrees)
    col = np.empty(rp[-1], dtype=np.int32)
    for v in range(N):
        d = int(degrees[v])
        col[rp[v]:rp[v + 1]] = np.sort(rng.choice(N, size=d, replace=False)) if d > 100 else np.unique(rng.integers(0, N, 4 * d))[:d]
    assert all(np.all(np.diff(col[rp[v]:rp[v + 1]]) > 0) for v in (0, 5, 300, 19999))
    dev = torch.device("cuda:0")
    rp_d, col_d = torch.from_numpy(rp).to(dev), torch.from_numpy(col).to(dev)
    T = np.sort(np.concatenate([np.fromiter(hubs, dtype=np.int64), 40 + 97 * np.arange(20)])).astype(np.int32)
    fanouts = (4000, 3)        # hop 1 takes most of the long rows
    ref_t, ref_h = oracle.vip(rp, col, T, 8, fanouts)
    t_np = [np.repeat(np.minimum(1.0, f / np.maximum(degrees, 1)).astype(np.float32), degrees) for f in fanouts]
    t_np[1] = (t_np[1] * rng.random(col.size)).astype(np.float32)
    p0 = np.zeros(N, np.float32)
    p0[T] = 8 / T.size
    gen_t, gen_h = oracle.vip_general(rp, col, p0, t_np, 2)
    for in_lists in (True, False):
        _say("long rows in the frontier, row blocks", in_lists)
        G = spp.Graph(ctx, rp_d, col_d, in_lists=in_lists, chunked=_CHUNKED)
        if in_lists:
            p, ph = spp.vip_propagate(ctx, G, torch.from_numpy(T).to(dev), 8, fanouts, per_hop=True)
            assert spp.vip_last_hops(ctx, 2)[0][0], "hop 1 was meant to be pushed"
            _check_vip(p, ref_t)
            _check_vip(ph[0], ref_h[0])
        pg, pgh = spp.vip_propagate_general(ctx, G, torch.from_numpy(p0).to(dev), [torch.from_numpy(a).to(dev) for a in t_np], 2,
                                            per_hop=True)
        _check_vip(pg, gen_t)
        _check_vip(pgh[0], gen_h[0])
        G.close()


def test_vip_chunked_layout_whole_blocks(spp, ctx, layout):
    """The chunked layout with more row blocks than CUs (257 blocks of 2^14 rows, 129 chunks of 2^15 sources):
    one workgroup then sums a whole row block and finishes its vertices itself.  Sparse (two or three
    out-edges per vertex) plus hub rows and hub columns, so that pieces are empty, tiny and large."""
    if layout != "chunked":
        pytest.skip("one layout only")
    rng = np.random.default_rng(2024)
    N = (1 << 22) + 1000
    deg = rng.integers(1, 4, N).astype(np.int64)
    deg[rng.integers(0, N, 2000)] = 0
    hubs = rng.integers(0, N, 12)
    deg[hubs] = rng.integers(3000, 9000, hubs.size)
    rp = np.zeros(N + 1, np.int64)
    rp[1:] = np.cumsum(deg)
    M = int(rp[-1])
    tgt = rng.integers(0, N, M).astype(np.int64)
    popular = rng.integers(0, N, 8)                        # columns that a tenth of the edges point at
    pick = rng.random(M) < 0.1
    tgt[pick] = popular[rng.integers(0, popular.size, int(pick.sum()))]
    # rows sorted and unique: sort by (row, target), drop repeats and self loops, rebuild the offsets
    row = np.repeat(np.arange(N, dtype=np.int64), deg)
    key = np.unique(row * N + tgt)
    row, tgt = key // N, key % N
    keep = row != tgt
    row, tgt = row[keep], tgt[keep]
    rp = np.zeros(N + 1, np.int64)
    np.add.at(rp, row + 1, 1)
    rp = np.cumsum(rp)
    col = tgt.astype(np.int32)
    dev = torch.device("cuda:0")
    G = spp.Graph(ctx, torch.from_numpy(rp).to(dev), torch.from_numpy(col).to(dev), in_lists=True, chunked=True)
    T = np.sort(np.concatenate([hubs, rng.choice(N, 200_000, replace=False)])).astype(np.int32)
    T = np.unique(T)
    fanouts = (4, 3, 2)
    _say("chunked layout, whole blocks: N", N, "M", col.size, "|T|", T.size)
    for include0 in (False, True):
        p, ph = spp.vip_propagate(ctx, G, torch.from_numpy(T).to(dev), 1024, fanouts, per_hop=True, include_hop0=include0)
        pushed, _ = spp.vip_last_hops(ctx, 3)
        assert not pushed[2], "the last hop was meant to be a dense one"
        ref_t, ref_h = oracle.vip(rp, col, T, 1024, fanouts, include_hop0=include0)
        _check_vip(p, ref_t)
        for h in range(3):
            _check_vip(ph[h], ref_h[h])
    G.close()


def _zipf_graph(rng, N, mean, hubs):
    """CSR with Zipf out-degrees scaled to `mean`, some empty rows and `hubs` rows of 4000+ entries; rows sorted, unique."""
    deg = rng.zipf(1.8, N).astype(np.int64)
    deg = np.minimum((deg * mean / deg.mean()).astype(np.int64), N // 3)
    deg[rng.integers(0, N, N // 20)] = 0
    for _ in range(hubs):
        deg[rng.integers(0, N)] = int(rng.integers(4000, min(N // 3, 20000)))
    rp = np.zeros(N + 1, np.int64)
    rp[1:] = np.cumsum(deg)
    col = np.empty(rp[-1], np.int32)
    for v in np.flatnonzero(deg):
        d = int(deg[v])
        if d > N // 8:
            row = rng.choice(N, d, replace=False)
        else:
            row = np.unique(rng.integers(0, N, 3 * d + 8))
            while row.size < d:
                row = np.unique(np.concatenate([row, rng.integers(0, N, 3 * d + 8)]))
            row = rng.permutation(row)[:d]
        col[rp[v]:rp[v + 1]] = np.sort(row)
    return rp, col


@pytest.mark.parametrize("case", range(8))
def test_random_shapes(spp, ctx, case):
    """Graph size, degree mix, number of hops, fanouts, batch and training-set sizes, row width, element
    type, cache size, number of id lists and fetch order drawn at random: all four calls (and the
    general propagation) against the oracle."""
    rng = np.random.default_rng(9000 + case)
    N = int(rng.choice([700, 5000, 17000, 40000, 70000]))
    rp, col = _zipf_graph(rng, N, float(rng.choice([3, 12, 40])), int(rng.integers(1, 4)) if N >= 40000 else 0)
    L = int(rng.integers(1, 4))
    fanouts = tuple(int(x) for x in rng.choice([1, 2, 5, 10, 15, 33, 64], L))
    B = int(rng.choice([1, 17, 256, 1024]))
    nT = int(min(N, rng.integers(B, 8 * B + 1)))
    T = np.sort(rng.choice(N, nT, replace=False)).astype(np.int32)
    K = int(rng.choice([2, 4, 8]))
    part = int(rng.integers(0, K))
    lo, hi = N * part // K, N * (part + 1) // K
    alpha = float(rng.choice([0.0, 0.05, 0.3, 1.0]))
    np_dt, D = [(np.float32, 100), (np.float32, 8), (np.float16, 128), (np.int16, 768)][int(rng.integers(0, 4))]   # int16: any 2-byte type
    _say("random shapes", case, "N", N, "M", col.size, "fanouts", fanouts, "B", B, "|T|", nT, "K", K, "part", part,
         "alpha", alpha, "D", D, np_dt.__name__)
    dev = torch.device("cuda:0")
    G = spp.Graph(ctx, torch.from_numpy(rp).to(dev), torch.from_numpy(col).to(dev), in_lists=True, chunked=_CHUNKED)
    # (1) vertex-inclusion probabilities, both entry points
    p, ph = spp.vip_propagate(ctx, G, torch.from_numpy(T).to(dev), B, fanouts, per_hop=True)
    rt, rh = oracle.vip(rp, col, T, B, fanouts)
    _check_vip(p, rt)
    for h in range(L):
        _check_vip(ph[h], rh[h])
    deg = np.diff(rp)
    t_np = [(rng.random(col.size) * np.repeat(np.minimum(1.0, f / np.maximum(deg, 1)), deg)).astype(np.float32) for f in fanouts]
    p0 = np.zeros(N, np.float32)
    p0[T] = rng.random(nT).astype(np.float32) * min(1.0, B / nT)
    pg, pgh = spp.vip_propagate_general(ctx, G, torch.from_numpy(p0).to(dev), [torch.from_numpy(a).to(dev) for a in t_np], L,
                                        per_hop=True)
    gt, gh = oracle.vip_general(rp, col, p0, t_np, L)
    _check_vip(pg, gt)
    for h in range(L):
        _check_vip(pgh[h], gh[h])
    # (2) cache by the propagated probabilities
    F = rng.integers(-30000, 30000, (N, D)).astype(np_dt)
    local = torch.from_numpy(F[lo:hi].copy()).to(dev)
    remote = torch.from_numpy(np.concatenate([F[:lo], F[hi:]])).pin_memory()
    cache = spp.build_vip_cache(ctx, p, lo, hi, K, alpha, remote, D, F.itemsize) if alpha > 0 else None
    ids_ref = oracle.cache_select(p.cpu().numpy(), lo, hi, K, alpha) if alpha > 0 else np.zeros(0, np.int32)
    if cache is not None:
        assert np.array_equal(cache.ids.cpu().numpy(), ids_ref)
    # (3) several minibatches with one set of launches
    nb = int(rng.integers(1, 6))
    items, refs = [], []
    for bi in range(nb):
        seeds = rng.permutation(T)[:int(rng.integers(1, min(B, nT) + 1))].astype(np.int32)
        items.append((torch.from_numpy(seeds).to(dev), 50 + bi, spp.MFGBuffers("cuda", B, fanouts, N)))
        refs.append(oracle.sample_mfg(rp, col, seeds, fanouts, 4242 + case, 50 + bi))
    spp.sample_mfg_multi(ctx, G, items, fanouts, 4242 + case)
    for (_, _, m), ref in zip(items, refs):
        _check_mfg(m, ref, L)
    # (4) their feature rows with one set of launches
    outs = [torch.full((max(ref.n[-1], 1) + 2, D), 7, dtype=local.dtype, device=dev) for ref in refs]
    lists = [(m.node_ids, ref.n[-1], None, o) for (_, _, m), ref, o in zip(items, refs, outs)]
    st = spp.gather_features_multi(ctx, cache, local, N, lo, hi, remote, lists, store_order=bool(rng.random() < 0.5))
    tot = [0, 0, 0]
    for ref, o in zip(refs, outs):
        want, _, counts = oracle.gather(N, lo, hi, F[lo:hi], F[ids_ref], ids_ref, remote.numpy(), ref.node_ids)
        assert np.array_equal(o[:ref.n[-1]].cpu().numpy(), want)
        assert bool((o[ref.n[-1]:] == 7).all())
        tot = [x + y for x, y in zip(tot, counts)]
    assert (st["n_local"], st["n_cache_hit"], st["n_miss"]) == tuple(tot)
    if cache is not None:
        cache.close()
    G.close()


# ----------------------------------------------------------------------------------------------
# Tiny config, all four calls
# ----------------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def tiny_case(spp, ctx, layout):
    _say("building Tiny")
    c = Case(spp, ctx, S.TINY)
    c.features()
    return c


def test_vip_tiny(spp, ctx, tiny_case):
    c = tiny_case
    cfg = c.cfg
    for name, T_d, T_h, B, fan in (("clamped p0", c.Tk_d, c.Tk, cfg.B, cfg.fanouts),
                                   ("global T", torch.from_numpy(c.T_all).cuda(), c.T_all, cfg.B, cfg.fanouts),
                                   ("tiny p0", torch.from_numpy(c.T_all).cuda(), c.T_all, 1, (2, 2, 2)),
                                   ("one hop", c.Tk_d, c.Tk, 16, (3,))):
        _say("vip tiny", name)
        p, ph = spp.vip_propagate(ctx, c.G, T_d, B, fan, per_hop=True)
        ref_t, ref_h = oracle.vip(c.rp, c.col, T_h, B, fan)
        _check_vip(p, ref_t)
        for h in range(len(fan)):
            _check_vip(ph[h], ref_h[h])


def test_cache_tiny(spp, ctx, tiny_case):
    c = tiny_case
    cfg = c.cfg
    p = spp.vip_propagate(ctx, c.G, c.Tk_d, cfg.B, cfg.fanouts)
    score = p.cpu().numpy()
    for alpha in (0.0, 0.05, cfg.alpha, 0.5, 3.0):
        _say("cache tiny alpha", alpha)
        cache = spp.build_vip_cache(ctx, p, c.lo, c.hi, cfg.K, alpha, c.remote, cfg.D, cfg.elem_bytes)
        ref = oracle.cache_select(score, c.lo, c.hi, cfg.K, alpha)
        assert np.array_equal(cache.ids.cpu().numpy(), ref)
        probe = torch.arange(cfg.N, dtype=torch.int32, device="cuda")
        slots = cache.lookup(probe).cpu().numpy()
        want = np.full(cfg.N, -1, dtype=np.int32)
        want[ref] = np.arange(ref.size)
        assert np.array_equal(slots, want)
        cache.close()
    # heavy ties and a degree-like score
    _say("cache tiny ties")
    deg = torch.from_numpy(np.bincount(c.col, minlength=cfg.N).astype(np.float32)).cuda()
    cache = spp.build_vip_cache(ctx, deg, c.lo, c.hi, cfg.K, 0.2, None, cfg.D, cfg.elem_bytes)
    assert np.array_equal(cache.ids.cpu().numpy(), oracle.cache_select(deg.cpu().numpy(), c.lo, c.hi, cfg.K, 0.2))
    cache.close()


def test_sample_and_gather_tiny(spp, ctx, tiny_case):
    c = tiny_case
    cfg = c.cfg
    p = spp.vip_propagate(ctx, c.G, c.Tk_d, cfg.B, cfg.fanouts)
    cache = spp.build_vip_cache(ctx, p, c.lo, c.hi, cfg.K, cfg.alpha, c.remote, cfg.D, cfg.elem_bytes)
    ids_ref = oracle.cache_select(p.cpu().numpy(), c.lo, c.hi, cfg.K, cfg.alpha)
    local = c.local_d.cpu().numpy()
    remote = c.remote.numpy()
    cache_rows = S.feature_rows(cfg, torch.from_numpy(ids_ref)).numpy()
    bufs = spp.MFGBuffers("cuda", cfg.B, cfg.fanouts, cfg.N)
    ctx.totals(reset=True)
    sums = dict(batches=0, n_nodes=0, n_edges=0, gather_calls=0, n_local=0, n_cache_hit=0, n_miss=0, n_local_host=0,
                n_miss_shared=0)
    for epoch in range(2):
        for bi, seeds in enumerate(S.epoch_batches(cfg, torch.from_numpy(c.Tk), epoch)):
            _say("tiny batch", epoch, bi, "seeds", seeds.numel())
            m = spp.sample_mfg(ctx, c.G, seeds.cuda(), cfg.fanouts, cfg.seed_sampler, epoch * 100 + bi, out=bufs)
            ref = oracle.sample_mfg(c.rp, c.col, seeds.numpy(), cfg.fanouts, cfg.seed_sampler, epoch * 100 + bi)
            _check_mfg(m, ref, cfg.L)
            out, stats = spp.gather_features(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, m.node_ids, n=m.n[-1])
            want, _, counts = oracle.gather(cfg.N, c.lo, c.hi, local, cache_rows, ids_ref, remote, ref.node_ids)
            assert np.array_equal(_bits(out.cpu().numpy()), _bits(want))
            assert (stats["n_local"], stats["n_cache_hit"], stats["n_miss"]) == counts
            assert stats["miss_bytes"] == counts[2] * cfg.D * cfg.elem_bytes
            for k, v in (("batches", 1), ("n_nodes", ref.n[-1]), ("n_edges", sum(ref.e)), ("gather_calls", 1),
                         ("n_local", counts[0]), ("n_cache_hit", counts[1]), ("n_miss", counts[2])):
                sums[k] += v
    assert ctx.totals() == sums
    # the same gather without a host round trip for the count, and with no cache at all
    m = spp.sample_mfg(ctx, c.G, torch.from_numpy(c.Tk[:100]).cuda(), (4, 3), 7, 3)
    out = torch.zeros((m.nb[-1], cfg.D), dtype=torch.float32, device="cuda")
    spp.gather_features(ctx, None, c.local_d, cfg.N, c.lo, c.hi, c.remote, m.node_ids, n=m.nb[-1],
                        n_device=m.n_final_device, out=out, sync=False)
    ctx.sync()
    st = spp.gather_last_stats(ctx)
    ids = m.node_ids[:m.n[-1]].cpu()
    assert torch.equal(out[:m.n[-1]].cpu(), S.feature_rows(cfg, ids))
    assert torch.all(out[m.n[-1]:] == 0)
    assert st["n_cache_hit"] == 0 and st["n_local"] + st["n_miss"] == m.n[-1]
    # device-time accounting: one piece per call and kind, shortest <= median <= longest
    ctx.timing(True)
    for _ in range(3):
        spp.gather_features(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, m.node_ids, n=m.n[-1])
    ms, cnt, shortest, median = ctx.time_stats()
    ctx.timing(False)
    for idx in (10, 11, 12):                     # hit copy, miss copy, classification
        longest = ms[idx] - shortest[idx] - median[idx]          # three pieces: the sum is shortest + median + longest
        assert cnt[idx] == 3 and 0 < shortest[idx] <= median[idx] <= longest + 1e-6
    assert cnt[9] == 0 and ms[9] == 0 and median[9] == 0
    assert ctx.times() == ([0.0] * 16, [0] * 16)
    cache.close()


def test_gather_edge_cases(spp, ctx, tiny_case):
    c = tiny_case
    cfg = c.cfg
    _say("gather: empty, duplicates, alpha sweep by limit")
    out, st = spp.gather_features(ctx, None, c.local_d, cfg.N, c.lo, c.hi, c.remote,
                                  torch.zeros(0, dtype=torch.int32, device="cuda"))
    assert out.shape[0] == 0 and st["n_local"] == st["n_miss"] == 0
    ids = torch.tensor([5, c.hi + 5, 5, cfg.N - 1, 0, c.hi], dtype=torch.int32, device="cuda")
    out, st = spp.gather_features(ctx, None, c.local_d, cfg.N, c.lo, c.hi, c.remote, ids)
    assert torch.equal(out.cpu(), S.feature_rows(cfg, ids.cpu()))
    assert (st["n_local"], st["n_cache_hit"], st["n_miss"]) == (3, 0, 3)
    p = spp.vip_propagate(ctx, c.G, c.Tk_d, cfg.B, cfg.fanouts)
    cache = spp.build_vip_cache(ctx, p, c.lo, c.hi, cfg.K, 0.5, c.remote, cfg.D, cfg.elem_bytes)
    allids = torch.arange(cfg.N, dtype=torch.int32, device="cuda")
    prev = -1
    for a in (0.0, 0.05, 0.1, 0.2, 0.5):
        cache.set_limit(min(cfg.cache_capacity(a), cache.n_cached))
        out, st = spp.gather_features(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, allids)
        ref_ids = oracle.cache_select(p.cpu().numpy(), c.lo, c.hi, cfg.K, a)
        assert st["n_cache_hit"] == ref_ids.size and st["n_cache_hit"] >= prev
        prev = st["n_cache_hit"]
        assert torch.equal(out.cpu(), S.feature_rows(cfg, allids.cpu()))
    cache.close()
    # bad ids are reported, not dereferenced
    with pytest.raises(spp.SppError):
        spp.gather_features(ctx, None, c.local_d, cfg.N, c.lo, c.hi, c.remote,
                            torch.tensor([1, cfg.N, -3], dtype=torch.int32, device="cuda"))
    # odd row width: 6-byte rows go through the 2-byte path
    loc = torch.arange(30, dtype=torch.int16, device="cuda").reshape(10, 3)
    rem = (1000 + torch.arange(90, dtype=torch.int16)).reshape(30, 3).pin_memory()
    ids = torch.tensor([0, 9, 10, 39, 3], dtype=torch.int32, device="cuda")
    out, st = spp.gather_features(ctx, None, loc, 40, 0, 10, rem, ids)
    full = torch.cat([loc.cpu(), rem])
    assert torch.equal(out.cpu(), full[ids.cpu().long()])
    # byte rows at an even address are served, an output at an odd address is refused
    loc8 = torch.arange(60, dtype=torch.uint8, device="cuda").reshape(10, 6)
    rem8 = (100 + torch.arange(180, dtype=torch.uint8)).reshape(30, 6).pin_memory()
    buf = torch.zeros(5 * 6 + 2, dtype=torch.uint8, device="cuda")
    out8, _ = spp.gather_features(ctx, None, loc8, 40, 0, 10, rem8, ids, out=buf[2:32].view(5, 6))
    assert torch.equal(out8.cpu(), torch.cat([loc8.cpu(), rem8])[ids.cpu().long()])
    with pytest.raises(spp.SppError):
        spp.gather_features(ctx, None, loc8, 40, 0, 10, rem8, ids, out=buf[1:31].view(5, 6))


def test_sample_multi_batches(spp, ctx, tiny_case):
    """Several minibatches in one set of launches: each equals the oracle's single-batch result."""
    c = tiny_case
    cfg = c.cfg
    _say("sample multi: 5 minibatches of 228, 1, 0, 100 and 37 seeds in one call")
    rng = np.random.default_rng(9)
    seeds = [c.Tk, c.Tk[:1], c.Tk[:0], rng.permutation(c.Tk)[:100], rng.permutation(c.Tk)[:37]]
    items = [(torch.from_numpy(np.ascontiguousarray(s_)).cuda(), 40 + k, spp.MFGBuffers("cuda", cfg.B, cfg.fanouts, cfg.N))
             for k, s_ in enumerate(seeds)]
    spp.sample_mfg_multi(ctx, c.G, items, cfg.fanouts, cfg.seed_sampler)
    for (sd, bi, m), s_ in zip(items, seeds):
        ref = oracle.sample_mfg(c.rp, c.col, s_, cfg.fanouts, cfg.seed_sampler, bi)
        _check_mfg(m, ref, cfg.L)
    with pytest.raises(spp.SppError):
        spp.sample_mfg_multi(ctx, c.G, items * 13, cfg.fanouts, cfg.seed_sampler)       # 65 minibatches
    _say("sample multi: 21, 40 and 64 minibatches in one call")
    for count in (21, 40, 64):
        seeds = [rng.permutation(c.Tk)[:rng.integers(1, 60)] for _ in range(count)]
        items = [(torch.from_numpy(np.ascontiguousarray(s_)).cuda(), 900 + k, spp.MFGBuffers("cuda", 64, cfg.fanouts, cfg.N))
                 for k, s_ in enumerate(seeds)]
        spp.sample_mfg_multi(ctx, c.G, items, cfg.fanouts, cfg.seed_sampler)
        for (sd, bi, m), s_ in zip(items, seeds):
            _check_mfg(m, oracle.sample_mfg(c.rp, c.col, s_, cfg.fanouts, cfg.seed_sampler, bi), cfg.L)


def test_sample_calls_that_reuse_and_change_their_buffers(spp, ctx, tiny_case):
    """The library keeps the per-minibatch pointers of a call on the device and stores them again only when
    a call brings other buffers: six buffer sets used in turn (more than it keeps), sets used with other seeds
    and minibatch numbers, with fewer minibatches, and a bad seed whose flag must not leak into later calls."""
    c = tiny_case
    cfg = c.cfg
    rng = np.random.default_rng(77)
    sets = [[spp.MFGBuffers("cuda", 64, cfg.fanouts, cfg.N) for _ in range(3)] for _ in range(6)]
    call = 0
    for rnd in range(3):
        for si in ([0, 1, 2, 3, 4, 5], [0, 1, 0, 1, 5, 0], [5, 4, 3, 2, 1, 0])[rnd]:
            count = 3 if (call % 4) else 2          # the same buffers, fewer minibatches
            seeds = [rng.permutation(c.Tk)[:rng.integers(0, 60)] for _ in range(count)]
            items = [(torch.from_numpy(np.ascontiguousarray(s_)).cuda(), 5000 + 7 * call + k, sets[si][k])
                     for k, s_ in enumerate(seeds)]
            _say("sample: call", call, "buffer set", si, "minibatches", count)
            spp.sample_mfg_multi(ctx, c.G, items, cfg.fanouts, cfg.seed_sampler, sync=bool(call % 2))
            ctx.sync()
            for (sd, bi, m), s_ in zip(items, seeds):
                cn = m.counts.cpu().numpy()
                m.n = [int(x) for x in cn[:cfg.L + 1]]
                m.e = [int(x) for x in cn[9:9 + cfg.L + 1]]
                _check_mfg(m, oracle.sample_mfg(c.rp, c.col, s_, cfg.fanouts, cfg.seed_sampler, bi), cfg.L)
            call += 1
    bad = torch.tensor([int(c.Tk[0]), cfg.N + 5], dtype=torch.int32, device="cuda")
    with pytest.raises(spp.SppError):
        spp.sample_mfg_multi(ctx, c.G, [(bad, 1, sets[0][0])], cfg.fanouts, cfg.seed_sampler)
    for k in range(3):                             # both sets of flags come round again: clean
        s_ = c.Tk[:10 + k]
        spp.sample_mfg_multi(ctx, c.G, [(torch.from_numpy(np.ascontiguousarray(s_)).cuda(), 9, sets[0][0])], cfg.fanouts, cfg.seed_sampler)
        _check_mfg(sets[0][0], oracle.sample_mfg(c.rp, c.col, s_, cfg.fanouts, cfg.seed_sampler, 9), cfg.L)


def test_gather_multi_lists(spp, ctx, tiny_case):
    """Several id lists in one call: same rows as one call per list, summed statistics."""
    c = tiny_case
    cfg = c.cfg
    _say("gather multi: lists of 0, 1, 2047, 2048, 2049 and 7000 ids, one with a device count")
    p = spp.vip_propagate(ctx, c.G, c.Tk_d, cfg.B, cfg.fanouts)
    cache = spp.build_vip_cache(ctx, p, c.lo, c.hi, cfg.K, cfg.alpha, c.remote, cfg.D, cfg.elem_bytes)
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    sizes = [0, 1, 2047, 2048, 2049, 7000]
    lists, singles, tot = [], [], dict(n_local=0, n_cache_hit=0, n_miss=0)
    for k, n in enumerate(sizes):
        ids = torch.randint(0, cfg.N, (n + 5,), device="cuda", generator=g, dtype=torch.int32)
        out = torch.zeros((n + 5, cfg.D), dtype=torch.float32, device="cuda")
        n_dev = torch.tensor([n], dtype=torch.int64, device="cuda") if k == 4 else None
        lists.append((ids, n + 5 if n_dev is not None else n, n_dev, out))
        ref, st = spp.gather_features(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, ids, n=n)
        singles.append(ref)
        for key in tot:
            tot[key] += st[key]
    st = spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists)
    assert {k: st[k] for k in tot} == tot
    # a remote vertex that several rows of the call miss crosses PCIe once: the other rows are copies
    all_ids = np.concatenate([l[0][:n0].cpu().numpy() for l, n0 in zip(lists, sizes)])
    cached = set(cache.ids.cpu().numpy().tolist())
    missed = np.array([g_ for g_ in all_ids if not (c.lo <= g_ < c.hi) and g_ not in cached])
    assert missed.size == tot["n_miss"]
    assert st["n_miss_shared"] == missed.size - np.unique(missed).size and st["n_miss_shared"] > 0
    assert st["miss_bytes"] == np.unique(missed).size * cfg.D * cfg.elem_bytes
    for (ids, n, n_dev, out), ref, n0 in zip(lists, singles, sizes):
        assert torch.equal(out[:n0], ref[:n0])
        assert torch.equal(out[:n0].cpu(), S.feature_rows(cfg, ids[:n0].cpu()))
        assert torch.all(out[n0:] == 0)
    with pytest.raises(spp.SppError):
        spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists * 11)   # 66 lists
    # maximal sharing: 64 lists of the same ids, no cache: every remote row but the first of a vertex is a copy
    _say("gather multi: 64 identical lists")
    ids = torch.randint(0, cfg.N, (3000,), device="cuda", generator=g, dtype=torch.int32)
    outs = [torch.zeros((3000, cfg.D), dtype=torch.float32, device="cuda") for _ in range(64)]
    st64 = spp.gather_features_multi(ctx, None, c.local_d, cfg.N, c.lo, c.hi, c.remote, [(ids, 3000, None, o) for o in outs])
    want = S.feature_rows(cfg, ids.cpu())
    for o in outs:
        assert torch.equal(o.cpu(), want)
    idn = ids.cpu().numpy()
    rem = idn[(idn < c.lo) | (idn >= c.hi)]
    assert st64["n_miss"] == 64 * rem.size and st64["n_miss_shared"] == 64 * rem.size - np.unique(rem).size
    # miss copy left running on the side stream while the stream samples the next minibatch, joined later
    _say("gather multi: deferred join")
    for (_, _, _, out) in lists:
        out.zero_()
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists, sync=False, join=False)
    m = spp.sample_mfg(ctx, c.G, torch.from_numpy(c.Tk[:64]).cuda(), (3, 2), 5, 1, sync=False)
    spp.gather_join(ctx)
    ctx.sync()
    for (ids, n, n_dev, out), n0 in zip(lists, sizes):
        assert torch.equal(out[:n0].cpu(), S.feature_rows(cfg, ids[:n0].cpu()))
    # and a second gather right after a deferred one joins by itself
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists[3:], sync=False, join=False)
    st2 = spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists[:3])
    assert st2["n_local"] + st2["n_cache_hit"] + st2["n_miss"] == sum(sizes[:3])
    # three unjoined gathers in a row, the middle one without rows: the third takes the workspace
    # of the first, so it must join the first itself; shared rows are copied at the join
    _say("gather multi: deferred joins around an empty call")
    for (_, _, _, out) in lists:
        out.zero_()
    same = [(lists[5][0], sizes[5], None, torch.zeros_like(lists[5][3])) for _ in range(3)]
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, same, sync=False, join=False)
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, [], sync=False, join=False)
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists, sync=False, join=False)
    ctx.sync()
    want5 = S.feature_rows(cfg, lists[5][0][:sizes[5]].cpu())
    for (_, _, _, out) in same:
        assert torch.equal(out[:sizes[5]].cpu(), want5)
    for (ids, n, n_dev, out), n0 in zip(lists, sizes):
        assert torch.equal(out[:n0].cpu(), S.feature_rows(cfg, ids[:n0].cpu()))
    # each call's miss copy queued before its hit copy: unjoined calls in a row, then a joined one
    _say("gather multi: hit copy beside the miss copy")
    for (_, _, _, out) in lists:
        out.zero_()
    twins = [(ids, n, n_dev, torch.zeros_like(out)) for (ids, n, n_dev, out) in lists]
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists, sync=False, join=False,
                              hit_beside_miss=True)
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, twins, sync=False, join=False,
                              hit_beside_miss=True, store_order=True)
    st3 = spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, same, hit_beside_miss=True)
    assert st3["n_local"] + st3["n_cache_hit"] + st3["n_miss"] == 3 * sizes[5]
    for group in (lists, twins):
        for (ids, n, n_dev, out), n0 in zip(group, sizes):
            assert torch.equal(out[:n0].cpu(), S.feature_rows(cfg, ids[:n0].cpu()))
    for (_, _, _, out) in same:
        assert torch.equal(out[:sizes[5]].cpu(), want5)
    cache.close()


def test_gather_in_store_order(spp, ctx, tiny_case):
    """Missed rows fetched in the order of the remote store: same rows and statistics as the hashed path,
    for several lists, one list with repeated ids, a split local store, unjoined calls in a row."""
    c = tiny_case
    cfg = c.cfg
    p = spp.vip_propagate(ctx, c.G, c.Tk_d, cfg.B, cfg.fanouts)
    cache = spp.build_vip_cache(ctx, p, c.lo, c.hi, cfg.K, cfg.alpha, c.remote, cfg.D, cfg.elem_bytes)
    g = torch.Generator(device="cuda")
    g.manual_seed(17)
    sizes = [0, 1, 2047, 2048, 2049, 7000, 3]
    lists = []
    for k, n in enumerate(sizes):
        ids = torch.randint(0, cfg.N, (n + 5,), device="cuda", generator=g, dtype=torch.int32)
        n_dev = torch.tensor([n], dtype=torch.int64, device="cuda") if k == 4 else None
        lists.append((ids, n + 5 if n_dev is not None else n, n_dev, torch.zeros((n + 5, cfg.D), dtype=torch.float32, device="cuda")))
    _say("store order: seven lists")
    ref = spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists)
    outs_ref = [l[3].clone() for l in lists]
    for l in lists:
        l[3].zero_()
    st = spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists, store_order=True)
    assert st == ref and st["n_miss_shared"] > 0
    for (ids, n, n_dev, out), want, n0 in zip(lists, outs_ref, sizes):
        assert torch.equal(out, want)
        assert torch.equal(out[:n0].cpu(), S.feature_rows(cfg, ids[:n0].cpu()))
        assert torch.all(out[n0:] == 0)
    _say("store order: one list, every id three times, no cache")
    ids = torch.randint(0, cfg.N, (1500,), device="cuda", generator=g, dtype=torch.int32).repeat(3)
    out, st1 = spp.gather_features(ctx, None, c.local_d, cfg.N, c.lo, c.hi, c.remote, ids, store_order=True)
    assert torch.equal(out.cpu(), S.feature_rows(cfg, ids.cpu()))
    idn = ids.cpu().numpy()
    rem = idn[(idn < c.lo) | (idn >= c.hi)]
    assert st1["n_miss"] == rem.size and st1["n_miss_shared"] == rem.size - np.unique(rem).size
    assert st1["miss_bytes"] == np.unique(rem).size * cfg.D * cfg.elem_bytes
    _say("store order: split local store, local rows from host memory beside the ordered remote rows")
    local_host = c.local_d.cpu().pin_memory()
    store = spp.build_local_store(ctx, p, c.lo, c.hi, 0.25, local_host)
    for l in lists:
        l[3].zero_()
    ref_s = spp.gather_features_multi(ctx, cache, store, cfg.N, c.lo, c.hi, c.remote, lists)
    for l in lists:
        l[3].zero_()
    st_s = spp.gather_features_multi(ctx, cache, store, cfg.N, c.lo, c.hi, c.remote, lists, store_order=True)
    assert st_s == ref_s and st_s["n_local_host"] > 0
    for (ids, n, n_dev, out), want in zip(lists, outs_ref):
        assert torch.equal(out, want)
    store.close()
    _say("store order: unjoined calls in a row, then a call without the flag")
    for l in lists:
        l[3].zero_()
    other = [(l[0], l[1], l[2], torch.zeros_like(l[3])) for l in lists]
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, lists, sync=False, join=False, store_order=True)
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, other, sync=False, join=False, store_order=True)
    third = [(l[0], l[1], l[2], torch.zeros_like(l[3])) for l in lists]
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, third, sync=False, join=False)
    ctx.sync()
    for group in (lists, other, third):
        for (ids, n, n_dev, out), want in zip(group, outs_ref):
            assert torch.equal(out, want)
    # nothing to order: no remote store and no remote id, an empty call
    loc_ids = torch.arange(c.lo, c.lo + 50, dtype=torch.int32, device="cuda")
    out, st0 = spp.gather_features(ctx, None, c.local_d, cfg.N, c.lo, c.hi, None, loc_ids, store_order=True)
    assert torch.equal(out, c.local_d[:50]) and st0["n_miss"] == 0
    spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, [], store_order=True)
    cache.close()


def test_local_store_tiny(spp, ctx, tiny_case):
    """VIP-ordered local storage: rank array, device prefix, and the gather with the local rows split
    between device and host (Sec. 3.2 on host-to-device transfers, Sec. 4.1)."""
    c = tiny_case
    cfg = c.cfg
    n_loc = c.hi - c.lo
    p = spp.vip_propagate(ctx, c.G, c.Tk_d, cfg.B, cfg.fanouts)
    score = p.cpu().numpy()
    local = c.local_d.cpu().numpy()
    local_host = c.local_d.cpu().pin_memory()
    remote = c.remote.numpy()
    cache = spp.build_vip_cache(ctx, p, c.lo, c.hi, cfg.K, cfg.alpha, c.remote, cfg.D, cfg.elem_bytes)
    ids_ref = oracle.cache_select(score, c.lo, c.hi, cfg.K, cfg.alpha)
    cache_rows = S.feature_rows(cfg, torch.from_numpy(ids_ref)).numpy()
    probe = torch.arange(-3, cfg.N + 3, dtype=torch.int32, device="cuda")
    seeds = S.epoch_batches(cfg, torch.from_numpy(c.Tk), 0)[0]
    ref = oracle.sample_mfg(c.rp, c.col, seeds.numpy(), cfg.fanouts, cfg.seed_sampler, 0)
    ids_d = torch.from_numpy(ref.node_ids).cuda()
    weird = score.copy()
    weird[c.lo:c.lo + 40:3] = -1.0
    weird[c.lo + 1:c.lo + 40:3] = np.nan
    weird[c.lo + 100:c.lo + 200] = 0.25                     # a run of ties
    for name, sc in (("vip", score), ("constant", np.full(cfg.N, 0.5, np.float32)), ("weird", weird)):
        rank_ref, order_ref = oracle.local_rank(sc, c.lo, c.hi)
        want_rank = np.full(probe.numel(), -1, dtype=np.int32)
        want_rank[3 + c.lo:3 + c.hi] = rank_ref
        for beta in (0.0, 0.05, 0.3, 1.0, 2.5):
            _say("local store", name, "beta", beta)
            store = spp.build_local_store(ctx, torch.from_numpy(sc).cuda(), c.lo, c.hi, beta, local_host)
            n_dev = oracle.local_capacity(beta, n_loc)
            assert store.n_device_rows == n_dev
            assert np.array_equal(store.rank(probe).cpu().numpy(), want_rank)
            out, stats = spp.gather_features(ctx, cache, store, cfg.N, c.lo, c.hi, c.remote, ids_d)
            want, _, counts = oracle.gather_split(cfg.N, c.lo, c.hi, local[order_ref[:n_dev]], local, rank_ref, n_dev,
                                                  cache_rows, ids_ref, remote, ref.node_ids)
            assert np.array_equal(_bits(out.cpu().numpy()), _bits(want))
            assert (stats["n_local"] - stats["n_local_host"], stats["n_cache_hit"], stats["n_miss"],
                    stats["n_local_host"]) == counts
            assert stats["miss_bytes"] == (counts[2] + counts[3]) * cfg.D * cfg.elem_bytes
            store.close()
    # a smaller beta is a prefix of a larger one: one store, limits set afterwards; running totals
    rank_ref, order_ref = oracle.local_rank(score, c.lo, c.hi)
    store = spp.build_local_store(ctx, p, c.lo, c.hi, 1.0, local_host)
    ctx.totals(reset=True)
    host_rows = 0
    for n_dev in (0, 1, 17, n_loc // 2, n_loc):
        store.set_limit(n_dev)
        out, stats = spp.gather_features(ctx, cache, store, cfg.N, c.lo, c.hi, c.remote, ids_d)
        want, _, counts = oracle.gather_split(cfg.N, c.lo, c.hi, local[order_ref[:n_dev]], local, rank_ref, n_dev,
                                              cache_rows, ids_ref, remote, ref.node_ids)
        assert np.array_equal(_bits(out.cpu().numpy()), _bits(want))
        assert stats["n_local_host"] == counts[3] and stats["n_miss"] == counts[2]
        host_rows += counts[3]
    t = ctx.totals()
    assert t["n_local_host"] == host_rows and t["gather_calls"] == 5
    with pytest.raises(spp.SppError):
        store.set_limit(n_loc + 1)
    # several lists in one call with the join deferred and no cache
    store.set_limit(n_loc // 5)
    n_dev = n_loc // 5
    lists, wants, tot = [], [], [0, 0, 0, 0]
    for j, take in enumerate((1, 700, 2049, 0, 5000)):
        ids = np.random.default_rng(j).integers(0, cfg.N, size=take).astype(np.int32)
        want, _, counts = oracle.gather_split(cfg.N, c.lo, c.hi, local[order_ref[:n_dev]], local, rank_ref, n_dev,
                                              None, None, remote, ids)
        out = torch.zeros((take + 2, cfg.D), dtype=torch.float32, device="cuda")
        lists.append((torch.from_numpy(ids).cuda(), take, None, out))
        wants.append(want)
        tot = [a + b for a, b in zip(tot, counts)]
    assert spp.gather_features_multi(ctx, None, store, cfg.N, c.lo, c.hi, c.remote, lists, sync=False, join=False) is None
    spp.gather_join(ctx)
    ctx.sync()
    st = spp.gather_last_stats(ctx)
    assert (st["n_local"] - st["n_local_host"], st["n_cache_hit"], st["n_miss"], st["n_local_host"]) == tuple(tot)
    for (ids, take, _, out), want in zip(lists, wants):
        assert np.array_equal(_bits(out[:take].cpu().numpy()), _bits(want))
        assert torch.all(out[take:] == 0)
    # local ids only and no remote store at all: the host-resident local rows are still served
    ids = np.arange(c.lo, c.hi, 7, dtype=np.int32)
    out, stats = spp.gather_features(ctx, None, store, cfg.N, c.lo, c.hi, None, torch.from_numpy(ids).cuda())
    assert np.array_equal(_bits(out.cpu().numpy()), _bits(local[ids - c.lo]))
    assert stats["n_miss"] == 0 and stats["n_local"] == ids.size and stats["n_local_host"] > 0
    # a remote id without a remote store is reported, its row left untouched, nothing else disturbed
    ids = np.array([c.lo, c.hi + 1 if c.hi + 1 < cfg.N else c.lo - 1, c.lo + 1], dtype=np.int32)
    out = torch.full((3, cfg.D), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(spp.SppError):
        spp.gather_features(ctx, None, store, cfg.N, c.lo, c.hi, None, torch.from_numpy(ids).cuda(), out=out)
    assert torch.all(out[1] == 7.0)
    assert np.array_equal(_bits(out[[0, 2]].cpu().numpy()), _bits(local[ids[[0, 2]] - c.lo]))
    # a store built for another range is refused
    with pytest.raises(spp.SppError):
        spp.gather_features(ctx, None, store, cfg.N, c.lo, c.hi - 1, c.remote, torch.from_numpy(ids).cuda())
    store.close()
    cache.close()
    # bfloat16 rows (2-byte elements): same split, same bytes
    half = c.local_d.to(torch.bfloat16)
    half_host = half.cpu().pin_memory()
    store = spp.build_local_store(ctx, p, c.lo, c.hi, 0.3, half_host)
    n_dev = oracle.local_capacity(0.3, n_loc)
    loc_ids = torch.arange(c.lo, c.hi, 3, dtype=torch.int32, device="cuda")
    out, stats = spp.gather_features(ctx, None, store, cfg.N, c.lo, c.hi, None, loc_ids)
    assert torch.equal(out.view(torch.int16).cpu(), half.view(torch.int16).cpu()[(loc_ids - c.lo).cpu().long()])
    on_dev = rank_ref[(loc_ids - c.lo).cpu().numpy()] < n_dev
    assert stats["n_local_host"] == int((~on_dev).sum())
    store.close()


def test_access_counts_and_empirical_policies_tiny(spp, ctx, tiny_case):
    """Empirical access frequencies (Sec. 3.2, "sim." and "oracle" policies): counts over sampled
    minibatches, bit for bit, and the caches ranked from them."""
    c = tiny_case
    cfg = c.cfg
    B, fanouts = 64, (5, 5)
    bufs = [spp.MFGBuffers("cuda", B, fanouts, cfg.N) for _ in range(4)]
    count_d = torch.zeros(cfg.N, dtype=torch.float32, device="cuda")
    count_ref = np.zeros(cfg.N, dtype=np.float32)
    for ep in range(3):
        perm = np.random.default_rng(50 + ep).permutation(c.Tk)
        groups = [perm[b:b + B] for b in range(0, perm.size - B + 1, B)]
        _say("access counts epoch", ep, "minibatches", len(groups))
        for g0 in range(0, len(groups), 4):
            grp = groups[g0:g0 + 4]
            items = [(torch.from_numpy(s_).cuda(), ep * 100 + g0 + k, bufs[k]) for k, s_ in enumerate(grp)]
            spp.sample_mfg_multi(ctx, c.G, items, fanouts, 11, sync=False)
            # counts read on the device: no host round trip between sampling and counting
            spp.access_count(ctx, [(bufs[k].node_ids, bufs[k].nb[-1], bufs[k].n_final_device) for k in range(len(grp))],
                             cfg.N, count_d, sync=(g0 == 0))
            for k, s_ in enumerate(grp):
                ref = oracle.sample_mfg(c.rp, c.col, s_, fanouts, 11, ep * 100 + g0 + k)
                oracle.access_count(cfg.N, ref.node_ids, count_ref)
    ctx.sync()
    assert np.array_equal(count_d.cpu().numpy(), count_ref)
    for alpha in (0.05, 0.3):
        cache = spp.build_vip_cache(ctx, count_d, c.lo, c.hi, cfg.K, alpha, None, cfg.D, cfg.elem_bytes)
        assert np.array_equal(cache.ids.cpu().numpy(), oracle.cache_select(count_ref, c.lo, c.hi, cfg.K, alpha))
        cache.close()
    # host counts, repeated ids (each appearance counts), an empty list, and ids out of range
    ids = torch.tensor([5, 5, 7, 5, cfg.N - 1], dtype=torch.int32, device="cuda")
    cnt = spp.access_count(ctx, [(ids, 5, None), (ids, 0, None), (ids, 3, None)], cfg.N)
    want = np.zeros(cfg.N, np.float32)
    want[5], want[7], want[cfg.N - 1] = 5, 2, 1
    assert np.array_equal(cnt.cpu().numpy(), want)
    bad = torch.tensor([1, -1, cfg.N, 2], dtype=torch.int32, device="cuda")
    cnt = torch.zeros(cfg.N, dtype=torch.float32, device="cuda")
    with pytest.raises(spp.SppError):
        spp.access_count(ctx, [(bad, 4, None)], cfg.N, cnt)
    assert cnt.sum().item() == 2 and cnt[1].item() == 1 and cnt[2].item() == 1


def _uniform_t(rp, f):
    d = np.diff(rp)
    return np.repeat(np.minimum(1.0, f / np.maximum(d, 1)).astype(np.float32), d)


def _general_caps(refs, L, slack=1.25):
    ncap = int(max(r.n[L] for r in refs) * slack) + 8
    ecaps = [int(max(r.e[h + 1] for r in refs) * slack) + 8 for h in range(L)]
    return ncap, ecaps


def test_general_probabilities_tiny(spp, ctx, tiny_case):
    """Proposition 1 with arbitrary initial and transition probabilities, and the sampler that takes
    every entry of a row with its own probability (Sec. 3.1, paragraph after Prop. 1)."""
    c = tiny_case
    cfg = c.cfg
    rng = np.random.default_rng(17)
    M = c.col.size
    t_np = [(rng.random(M) * 0.6).astype(np.float32), (rng.random(M) ** 3).astype(np.float32),
            np.where(rng.random(M) < 0.1, 1.0, rng.random(M) * 0.2).astype(np.float32)]
    t_d = [torch.from_numpy(a).cuda() for a in t_np]
    p0 = np.where(rng.random(cfg.N) < 0.05, rng.random(cfg.N), 0.0).astype(np.float32)
    p0[:3] = [1.0, 0.0, 0.5]
    # a graph with the row-block structure takes the binned push, one without it the atomic push
    G_plain = spp.Graph(ctx, c.rowptr_d, c.col_d, in_lists=False)
    for L, hop0 in ((3, False), (2, True), (1, False)):
        rt, rh = oracle.vip_general(c.rp, c.col, p0, t_np[:L], L, include_hop0=hop0)
        for G in (c.G, G_plain):
            _say("general vip L", L, "hop0", hop0, "row blocks", G is c.G)
            p, ph = spp.vip_propagate_general(ctx, G, torch.from_numpy(p0).cuda(), t_d[:L], L, per_hop=True, include_hop0=hop0)
            _check_vip(p, rt)
            for h in range(L):
                _check_vip(ph[h], rh[h])
    # degenerate inputs: nobody in the minibatch (empty frontier at every hop); nothing ever sampled
    for G in (c.G, G_plain):
        _say("general vip, empty frontier / zero transitions, row blocks", G is c.G)
        z, zh = spp.vip_propagate_general(ctx, G, torch.zeros(cfg.N, device="cuda"), t_d[:2], 2, per_hop=True)
        assert not bool(z.any()) and not bool(zh.any())
        zt = torch.zeros(M, device="cuda")
        p, ph = spp.vip_propagate_general(ctx, G, torch.from_numpy(p0).cuda(), zt, 2, per_hop=True, include_hop0=True)
        assert not bool(ph.any())
        _check_vip(p, oracle.vip_general(c.rp, c.col, p0, np.zeros(M, np.float32), 2, include_hop0=True)[0])
    # one tensor for every hop; the uniform instantiation agrees with the uniform entry point
    _say("general vip, uniform instantiation")
    p0u = np.zeros(cfg.N, np.float32)
    p0u[c.Tk] = min(1.0, cfg.B / c.Tk.size)
    tu = [_uniform_t(c.rp, f) for f in cfg.fanouts]
    pg = spp.vip_propagate_general(ctx, c.G, torch.from_numpy(p0u).cuda(), [torch.from_numpy(a).cuda() for a in tu], cfg.L)
    _check_vip(pg, oracle.vip(c.rp, c.col, c.Tk, cfg.B, cfg.fanouts)[0])
    one = spp.vip_propagate_general(ctx, c.G, torch.from_numpy(p0).cuda(), t_d[0], 2)
    _check_vip(one, oracle.vip_general(c.rp, c.col, p0, t_np[0], 2)[0])
    # a probability outside [0, 1] is reported and taken as 0
    bad_t = t_np[0].copy()
    bad_t[5] = 1.5
    bad_t[9] = np.nan
    with pytest.raises(spp.SppError):
        spp.vip_propagate_general(ctx, c.G, torch.from_numpy(p0).cuda(), torch.from_numpy(bad_t).cuda(), 1)
    bad_p = p0.copy()
    bad_p[7] = -0.5
    with pytest.raises(spp.SppError):
        spp.vip_propagate_general(ctx, c.G, torch.from_numpy(bad_p).cuda(), t_d[0], 1)

    # ---- the sampler
    batches = S.epoch_batches(cfg, torch.from_numpy(c.Tk), 0)
    seeds_list = [b.numpy() for b in batches[:2]] + [c.Tk[:7], np.array([], dtype=np.int32)]
    for L in (3, 1):
        refs = [oracle.sample_mfg_general(c.rp, c.col, t_np[:L], s_, L, 99, 40 + j) for j, s_ in enumerate(seeds_list)]
        ncap, ecaps = _general_caps(refs, L)
        _say("general sampler L", L, "caps", ncap, ecaps)
        bufs = [spp.MFGBuffers("cuda", 0, (), cfg.N, capacities=(ncap, ecaps)) for _ in seeds_list]
        items = [(torch.from_numpy(s_).cuda(), 40 + j, bufs[j]) for j, s_ in enumerate(seeds_list)]
        spp.sample_mfg_general(ctx, c.G, t_d[:L], items, L, 99)
        for b, ref in zip(bufs, refs):
            _check_mfg(b, ref, L)
    # t = 1 everywhere: full expansion; t = 0: nothing beyond the seeds
    ones = torch.ones(M, dtype=torch.float32, device="cuda")
    ref = oracle.sample_mfg_general(c.rp, c.col, np.ones(M, np.float32), c.Tk[:5], 2, 1, 0)
    b = spp.MFGBuffers("cuda", 0, (), cfg.N, capacities=(ref.n[2], [ref.e[1], ref.e[2]]))      # exact capacities suffice
    spp.sample_mfg_general(ctx, c.G, ones, [(torch.from_numpy(c.Tk[:5]).cuda(), 0, b)], 2, 1)
    _check_mfg(b, ref, 2)
    spp.sample_mfg_general(ctx, c.G, torch.zeros_like(ones), [(torch.from_numpy(c.Tk[:5]).cuda(), 0, b)], 2, 1)
    assert b.n == [5, 5, 5] and b.e == [0, 0, 0]
    # capacities one short, for the edges of hop 2 and for the ids: reported, nothing written out of bounds
    # (the buffers are followed by a guard that must stay untouched), and the next call is not affected
    for ncap, ecaps in ((ref.n[2], [ref.e[1], ref.e[2] - 1]), (ref.n[2] - 1, [ref.e[1], ref.e[2]])):
        small = spp.MFGBuffers("cuda", 0, (), cfg.N, capacities=(ncap, ecaps))
        ok = spp.MFGBuffers("cuda", 0, (), cfg.N, capacities=(ref.n[2] + 3, [ref.e[1] + 3, ref.e[2] + 3]))
        ok.node_ids.fill_(-7)
        with pytest.raises(spp.SppError):
            spp.sample_mfg_general(ctx, c.G, ones, [(torch.from_numpy(c.Tk[:5]).cuda(), 0, small),
                                                    (torch.from_numpy(c.Tk[:5]).cuda(), 0, ok)], 2, 1)
        # the minibatch that fitted is complete and correct
        ctx.sync()
        cnt = ok.counts.cpu().numpy()
        assert cnt[2] == ref.n[2] and np.array_equal(ok.node_ids[:ref.n[2]].cpu().numpy(), ref.node_ids)
        assert torch.all(ok.node_ids[ref.n[2]:] == -7)
    spp.sample_mfg_general(ctx, c.G, ones, [(torch.from_numpy(c.Tk[:5]).cuda(), 0, b)], 2, 1)
    _check_mfg(b, ref, 2)
    # the fanout sampler after the general one on the same context (shared workspaces)
    m = spp.sample_mfg(ctx, c.G, torch.from_numpy(seeds_list[0]).cuda(), cfg.fanouts, cfg.seed_sampler, 0)
    _check_mfg(m, oracle.sample_mfg(c.rp, c.col, seeds_list[0], cfg.fanouts, cfg.seed_sampler, 0), cfg.L)


# ----------------------------------------------------------------------------------------------
# scaled copies of the other configs: several tiles, ragged tails, hubs, 16-bit rows
# ----------------------------------------------------------------------------------------------

SCALED = [
    ("mid", S.scaled(S.MID, 150_000)),
    ("large", S.scaled(S.LARGE, 200_000)),
    ("wide", S.scaled(S.WIDE, 200_000, pop_cap=20_000)),
    ("skew", S.scaled(S.SKEW, 1 << 17)),
]


@pytest.mark.parametrize("name,cfg", SCALED, ids=[n for n, _ in SCALED])
def test_scaled_config_end_to_end(spp, ctx, name, cfg):
    _say("scaled", name, "N", cfg.N)
    c = Case(spp, ctx, cfg, gen_device="cuda")
    _say("graph M", c.M, "max in-degree", int(np.bincount(c.col, minlength=cfg.N).max()), "|T_k|", c.Tk.size)
    c.features()
    p, ph = spp.vip_propagate(ctx, c.G, c.Tk_d, cfg.B, cfg.fanouts, per_hop=True)
    ref_t, ref_h = oracle.vip(c.rp, c.col, c.Tk, cfg.B, cfg.fanouts)
    _check_vip(p, ref_t)
    for h in range(cfg.L):
        _check_vip(ph[h], ref_h[h])
    _say("vip ok")
    cache = spp.build_vip_cache(ctx, p, c.lo, c.hi, cfg.K, cfg.alpha, c.remote, cfg.D, cfg.elem_bytes)
    ids_ref = oracle.cache_select(p.cpu().numpy(), c.lo, c.hi, cfg.K, cfg.alpha)
    assert np.array_equal(cache.ids.cpu().numpy(), ids_ref)
    _say("cache ok", ids_ref.size)
    # end to end: oracle p -> oracle cache differs from the GPU's only at scores within tolerance of the cut
    ids_o = oracle.cache_select(ref_t.astype(np.float32), c.lo, c.hi, cfg.K, cfg.alpha)
    diff = np.setxor1d(ids_o, ids_ref)
    if diff.size:
        cut = ref_t[ids_o[-1]]
        assert np.all(np.abs(ref_t[diff] - cut) <= 1e-5 * cut)
    local = _np(c.local_d)
    remote = _np(c.remote)
    cache_rows = _np(S.feature_rows(cfg, torch.from_numpy(ids_ref)))
    bufs = spp.MFGBuffers("cuda", cfg.B, cfg.fanouts, cfg.N)
    batches = S.epoch_batches(cfg, torch.from_numpy(c.Tk), 0)
    for bi, seeds in enumerate(batches[:2] + batches[-1:]):
        _say("batch", bi, "seeds", seeds.numel())
        m = spp.sample_mfg(ctx, c.G, seeds.cuda(), cfg.fanouts, cfg.seed_sampler, bi, out=bufs)
        ref = oracle.sample_mfg(c.rp, c.col, seeds.numpy(), cfg.fanouts, cfg.seed_sampler, bi)
        _check_mfg(m, ref, cfg.L)
        out, stats = spp.gather_features(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote, m.node_ids, n=m.n[-1])
        want, _, counts = oracle.gather(cfg.N, c.lo, c.hi, local, cache_rows, ids_ref, remote, ref.node_ids)
        assert np.array_equal(_bits(_np(out)), _bits(want))
        assert (stats["n_local"], stats["n_cache_hit"], stats["n_miss"]) == counts
    # the same minibatches through the batched calls, misses fetched in store order (this workload's row width and type)
    _say("batched calls, store order")
    group = batches[:2] + batches[-1:]
    mb = [spp.MFGBuffers("cuda", cfg.B, cfg.fanouts, cfg.N) for _ in group]
    spp.sample_mfg_multi(ctx, c.G, [(s_.cuda(), bi, mb[bi]) for bi, s_ in enumerate(group)], cfg.fanouts, cfg.seed_sampler, sync=False)
    outs = [torch.zeros((b_.nb[-1], cfg.D), dtype=cfg.torch_dtype, device="cuda") for b_ in mb]
    st = spp.gather_features_multi(ctx, cache, c.local_d, cfg.N, c.lo, c.hi, c.remote,
                                   [(b_.node_ids, b_.nb[-1], b_.n_final_device, o_) for b_, o_ in zip(mb, outs)], store_order=True)
    tot = [0, 0, 0]
    ids_all = []
    for bi, (seeds, b_, o_) in enumerate(zip(group, mb, outs)):
        ref = oracle.sample_mfg(c.rp, c.col, seeds.numpy(), cfg.fanouts, cfg.seed_sampler, bi)
        want, tag, counts = oracle.gather(cfg.N, c.lo, c.hi, local, cache_rows, ids_ref, remote, ref.node_ids)
        assert np.array_equal(_bits(_np(o_[:ref.n[-1]])), _bits(want))
        assert not bool(o_[ref.n[-1]:].any())
        tot = [x + y for x, y in zip(tot, counts)]
        ids_all.append(ref.node_ids[tag == 2])
    assert (st["n_local"], st["n_cache_hit"], st["n_miss"]) == tuple(tot)
    missed = np.concatenate(ids_all)
    assert st["n_miss_shared"] == missed.size - np.unique(missed).size
    # general probabilities on the same graph: hub rows span many 64-entry chunks of the sampler's ballots
    _say("general probabilities")
    rng = np.random.default_rng(5)
    t_np = (rng.random(c.col.size) * np.repeat(np.minimum(1.0, 6.0 / np.maximum(np.diff(c.rp), 1)), np.diff(c.rp))).astype(np.float32)
    t_d = torch.from_numpy(t_np).cuda()
    p0 = np.zeros(cfg.N, np.float32)
    p0[c.Tk] = min(1.0, cfg.B / c.Tk.size)
    pg, pgh = spp.vip_propagate_general(ctx, c.G, torch.from_numpy(p0).cuda(), t_d, 2, per_hop=True)
    rt, rh = oracle.vip_general(c.rp, c.col, p0, t_np, 2)
    _check_vip(pg, rt)
    _check_vip(pgh[1], rh[1])
    grefs = [oracle.sample_mfg_general(c.rp, c.col, t_np, s_.numpy(), 2, 3, bi) for bi, s_ in enumerate(batches[:2])]
    ncap, ecaps = _general_caps(grefs, 2)
    gb = [spp.MFGBuffers("cuda", 0, (), cfg.N, capacities=(ncap, ecaps)) for _ in grefs]
    spp.sample_mfg_general(ctx, c.G, t_d, [(s_.cuda(), bi, gb[bi]) for bi, s_ in enumerate(batches[:2])], 2, 3)
    for b_, r_ in zip(gb, grefs):
        _check_mfg(b_, r_, 2)
    # the same batches with the local rows split between device and host (10 % on the device)
    _say("local store")
    local_host = c.local_d.cpu().pin_memory()
    store = spp.build_local_store(ctx, p, c.lo, c.hi, 0.1, local_host)
    rank_ref, order_ref = oracle.local_rank(p.cpu().numpy(), c.lo, c.hi)
    n_dev = oracle.local_capacity(0.1, c.hi - c.lo)
    assert store.n_device_rows == n_dev
    probe = torch.arange(c.lo, c.hi, dtype=torch.int32, device="cuda")
    assert np.array_equal(store.rank(probe).cpu().numpy(), rank_ref)
    for bi, seeds in enumerate(batches[:2] + batches[-1:]):
        ref = oracle.sample_mfg(c.rp, c.col, seeds.numpy(), cfg.fanouts, cfg.seed_sampler, bi)
        ids_d = torch.from_numpy(ref.node_ids).cuda()
        out, stats = spp.gather_features(ctx, cache, store, cfg.N, c.lo, c.hi, c.remote, ids_d)
        want, _, counts = oracle.gather_split(cfg.N, c.lo, c.hi, local[order_ref[:n_dev]], local, rank_ref, n_dev,
                                              cache_rows, ids_ref, remote, ref.node_ids)
        assert np.array_equal(_bits(_np(out)), _bits(want))
        assert (stats["n_local"] - stats["n_local_host"], stats["n_cache_hit"], stats["n_miss"],
                stats["n_local_host"]) == counts
    store.close()
    cache.close()
    c.G.close()
