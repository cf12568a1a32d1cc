"""Parity at the full size of the Mid workload (2.4M vertices, ~121M edges, fp32 D=100, K=8,
alpha=0.16), in the launch configuration bench.py times: two minibatches in flight on two
contexts, asynchronous calls, |S_L| read on the device by the gather."""
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

    _say("batches, two in flight")
    batches = S.epoch_batches(cfg, Tk, 0)[:6]
    lanes = []
    for k in range(2):
        c = ctx if k == 0 else spp.Context(0, stream=torch.cuda.Stream(dev))
        b = spp.MFGBuffers(dev, cfg.B, cfg.fanouts, cfg.N)
        lanes.append((c, b, torch.zeros((b.nb[-1], cfg.D), dtype=cfg.torch_dtype, device=dev)))
    torch.cuda.synchronize()
    local_np, remote_np = local.cpu().numpy(), remote.numpy()
    for r in range(0, len(batches), 2):
        for k in range(2):
            c, b, o = lanes[k]
            spp.sample_mfg(c, G, batches[r + k], cfg.fanouts, cfg.seed_sampler, r + k, out=b, sync=False)
            spp.gather_features(c, cache, local, cfg.N, lo, hi, remote, b.node_ids, n=b.nb[-1],
                                n_device=b.n_final_device, out=o, sync=False)
        for k in range(2):
            c, b, o = lanes[k]
            c.sync()
            st = spp.gather_last_stats(c)
            counts = b.counts.cpu().numpy()
            ref = oracle.sample_mfg(rp, col, batches[r + k].cpu().numpy(), cfg.fanouts, cfg.seed_sampler, r + k)
            n = [int(x) for x in counts[:cfg.L + 1]]
            e = [int(x) for x in counts[9:9 + cfg.L + 1]]
            _say("batch", r + k, "n", n, "e", e)
            assert n == ref.n and e == ref.e
            assert np.array_equal(b.node_ids[:n[-1]].cpu().numpy(), ref.node_ids)
            for h in range(cfg.L):
                assert np.array_equal(b.indptr[h][:n[h] + 1].cpu().numpy(), ref.indptr[h])
                assert np.array_equal(b.src[h][:e[h + 1]].cpu().numpy(), ref.src[h])
            want, _, cnt = oracle.gather(cfg.N, lo, hi, local_np, cache_rows, ids_ref, remote_np, ref.node_ids)
            assert np.array_equal(o[:n[-1]].cpu().numpy().view(np.uint32), want.view(np.uint32))
            assert (st["n_local"], st["n_cache_hit"], st["n_miss"]) == cnt
    for c, _, _ in lanes[1:]:
        c.close()
    cache.close()
    G.close()
    ctx.close()
