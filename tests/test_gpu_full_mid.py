"""Parity at the full size of the Mid workload (2.4M vertices, ~121M edges, fp32 D=100, K=8,
alpha=0.16), in the launch configuration bench.py times: groups of 64 minibatches sampled by one
call and gathered by one set of launches, asynchronous calls with the join of the miss copy
deferred, |S_L| read on the device; then the local-storage split, the access counts and the
general-probability entry points at the same size."""
import numpy as np
import pytest
import torch

import oracle
from workloads import synth as S

pytestmark = pytest.mark.gpu


def _say(*a):
    print("[case]", *a, flush=True)


def test_mid_full_size():
    import paper_2305_03152_amd as spp
    cfg = S.MID
    dev = torch.device("cuda:0")
    lo, hi = cfg.bounds()
    _say("mid full: generating")
    g = S.make_graph(cfg, dev)
    T = S.make_training_set(cfg, dev)
    Tk = S.local_training_set(cfg, T)
    rp, col = g.rowptr.cpu().numpy(), g.col.cpu().numpy()
    _say("N", g.N, "M", g.M, "|T_k|", Tk.numel())
    ctx = spp.Context(0)
    G = spp.Graph(ctx, g.rowptr, g.col, in_lists=True)

    _say("vip")
    p, ph = spp.vip_propagate(ctx, G, Tk, cfg.B, cfg.fanouts, per_hop=True)
    ref_t, ref_h = oracle.vip(rp, col, Tk.cpu().numpy(), cfg.B, cfg.fanouts)
    for name, a, b in [("total", p, ref_t)] + [(f"hop{h + 1}", ph[h], ref_h[h]) for h in range(cfg.L)]:
        a = a.cpu().numpy().astype(np.float64)
        bad = np.flatnonzero(np.abs(a - b) > 1e-5 * b + 1e-37)
        assert bad.size == 0, (name, bad[:5], a[bad[:5]], b[bad[:5]])
        assert np.all(a[b == 0] == 0)

    _say("features")
    local = S.feature_block(cfg, lo, hi, dev)
    nrem = cfg.N - (hi - lo)
    remote = torch.empty((nrem, cfg.D), dtype=cfg.torch_dtype).pin_memory()
    for a in range(0, nrem, 1 << 19):
        b = min(nrem, a + (1 << 19))
        remote[a:b].copy_(S.feature_rows(cfg, S.remote_ids(cfg, a, b, dev)))
    torch.cuda.synchronize()

    _say("cache")
    cache = spp.build_vip_cache(ctx, p, lo, hi, cfg.K, cfg.alpha, remote, cfg.D, cfg.elem_bytes)
    ids_ref = oracle.cache_select(p.cpu().numpy(), lo, hi, cfg.K, cfg.alpha)
    assert np.array_equal(cache.ids.cpu().numpy(), ids_ref) and ids_ref.size == cfg.cache_capacity()
    cache_rows = S.feature_rows(cfg, torch.from_numpy(ids_ref)).numpy()

    _say("batches: groups of 64 per call, join deferred, two buffer sets (the benchmark's launch configuration)")
    G8 = 64
    batches = [b for ep in range(6) for b in S.epoch_batches(cfg, Tk, ep)][:2 * G8]       # 24 per epoch
    assert len(batches) == 2 * G8
    sets = []
    for _ in range(2):
        b = [spp.MFGBuffers(dev, cfg.B, cfg.fanouts, cfg.N) for _ in range(G8)]
        o = [torch.zeros((b[0].nb[-1], cfg.D), dtype=cfg.torch_dtype, device=dev) for _ in range(G8)]
        sets.append((b, o))
    count_d = torch.zeros(cfg.N, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    local_np, remote_np = local.cpu().numpy(), remote.numpy()
    ctx.totals(reset=True)
    for gi in range(2):
        b, o = sets[gi]
        idx = range(gi * G8, (gi + 1) * G8)
        spp.sample_mfg_multi(ctx, G, [(batches[i], i, b[k]) for k, i in enumerate(idx)], cfg.fanouts, cfg.seed_sampler,
                             sync=False)
        spp.access_count(ctx, [(b[k].node_ids, b[k].nb[-1], b[k].n_final_device) for k in range(G8)], cfg.N, count_d,
                         sync=False)
        spp.gather_join(ctx)
        spp.gather_features_multi(ctx, cache, local, cfg.N, lo, hi, remote,
                                  [(b[k].node_ids, b[k].nb[-1], b[k].n_final_device, o[k]) for k in range(G8)],
                                  sync=False, join=False, store_order=(gi == 1),     # both miss orders
                                  hit_beside_miss=(gi == 1))                         # and both orders of the copies
    spp.gather_join(ctx)
    ctx.sync()
    count_ref = np.zeros(cfg.N, dtype=np.float32)
    tot = dict(n_local=0, n_cache_hit=0, n_miss=0)
    refs = []
    for gi in range(2):
        b, o = sets[gi]
        for k in range(G8):
            i = gi * G8 + k
            counts = b[k].counts.cpu().numpy()
            ref = oracle.sample_mfg(rp, col, batches[i].cpu().numpy(), cfg.fanouts, cfg.seed_sampler, i)
            refs.append(ref)
            n = [int(x) for x in counts[:cfg.L + 1]]
            e = [int(x) for x in counts[9:9 + cfg.L + 1]]
            _say("batch", i, "n", n, "e", e)
            assert n == ref.n and e == ref.e
            assert np.array_equal(b[k].node_ids[:n[-1]].cpu().numpy(), ref.node_ids)
            for h in range(cfg.L):
                assert np.array_equal(b[k].indptr[h][:n[h] + 1].cpu().numpy(), ref.indptr[h])
                assert np.array_equal(b[k].src[h][:e[h + 1]].cpu().numpy(), ref.src[h])
            want, _, cnt = oracle.gather(cfg.N, lo, hi, local_np, cache_rows, ids_ref, remote_np, ref.node_ids)
            assert np.array_equal(o[k][:n[-1]].cpu().numpy().view(np.uint32), want.view(np.uint32))
            for key, v in zip(("n_local", "n_cache_hit", "n_miss"), cnt):
                tot[key] += v
            oracle.access_count(cfg.N, ref.node_ids, count_ref)
    t = ctx.totals()
    assert (t["n_local"], t["n_cache_hit"], t["n_miss"]) == (tot["n_local"], tot["n_cache_hit"], tot["n_miss"])
    assert t["batches"] == 2 * G8 and t["gather_calls"] == 2
    assert np.array_equal(count_d.cpu().numpy(), count_ref)

    _say("local rows split between device and host (beta = 0.1)")
    local_host = local.cpu().pin_memory()
    store = spp.build_local_store(ctx, p, lo, hi, 0.1, local_host)
    rank_ref, order_ref = oracle.local_rank(p.cpu().numpy(), lo, hi)
    n_dev = oracle.local_capacity(0.1, hi - lo)
    assert store.n_device_rows == n_dev
    assert np.array_equal(store.rank(torch.arange(lo, hi, dtype=torch.int32, device=dev)).cpu().numpy(), rank_ref)
    b, o = sets[0]
    st = spp.gather_features_multi(ctx, cache, store, cfg.N, lo, hi, remote,
                                   [(b[k].node_ids, b[k].nb[-1], b[k].n_final_device, o[k]) for k in range(G8)])
    sums = [0, 0, 0, 0]
    dev_rows = local_np[order_ref[:n_dev]]
    for k in range(G8):
        ref = refs[k]
        want, _, cnt = oracle.gather_split(cfg.N, lo, hi, dev_rows, local_np, rank_ref, n_dev, cache_rows, ids_ref,
                                           remote_np, ref.node_ids)
        assert np.array_equal(o[k][:ref.n[-1]].cpu().numpy().view(np.uint32), want.view(np.uint32))
        sums = [x + y for x, y in zip(sums, cnt)]
    assert (st["n_local"] - st["n_local_host"], st["n_cache_hit"], st["n_miss"], st["n_local_host"]) == tuple(sums)
    store.close()

    _say("general probabilities: propagation and sampler")
    rng = np.random.default_rng(8)
    deg = np.diff(rp)
    t_np = (rng.random(col.size) * np.repeat(np.minimum(1.0, 8.0 / np.maximum(deg, 1)), deg)).astype(np.float32)
    t_d = torch.from_numpy(t_np).to(dev)
    p0 = np.zeros(cfg.N, np.float32)
    p0[Tk.cpu().numpy()] = cfg.B / Tk.numel()
    pg = spp.vip_propagate_general(ctx, G, torch.from_numpy(p0).to(dev), t_d, 2)
    rg, _ = oracle.vip_general(rp, col, p0, t_np, 2)
    a = pg.cpu().numpy().astype(np.float64)
    bad = np.flatnonzero(np.abs(a - rg) > 1e-5 * rg + 1e-37)
    assert bad.size == 0, (bad[:5], a[bad[:5]], rg[bad[:5]])
    grefs = [oracle.sample_mfg_general(rp, col, t_np, batches[i].cpu().numpy(), 2, 4, i) for i in range(2)]
    ncap = int(max(r.n[2] for r in grefs) * 1.2)
    ecaps = [int(max(r.e[h + 1] for r in grefs) * 1.2) for h in range(2)]
    gb = [spp.MFGBuffers(dev, 0, (), cfg.N, capacities=(ncap, ecaps)) for _ in grefs]
    spp.sample_mfg_general(ctx, G, t_d, [(batches[i], i, gb[i]) for i in range(2)], 2, 4)
    for b_, r_ in zip(gb, grefs):
        assert b_.n == r_.n and b_.e == r_.e
        assert np.array_equal(b_.node_ids[:r_.n[2]].cpu().numpy(), r_.node_ids)
        for h in range(2):
            assert np.array_equal(b_.src[h][:r_.e[h + 1]].cpu().numpy(), r_.src[h])
    cache.close()
    G.close()
    ctx.close()
