#!/usr/bin/env python3
"""Benchmark of the per-partition data path on one MI355X.

A step is one minibatch through the per-batch rows of the path: multi-hop fanout sampling into
MFGs, then the cache-aware feature gather of |S_L| rows (local shard / VIP cache in HBM, misses
from pinned host memory on a side stream).  The one-time rows (VIP propagation, cache ranking and
fill) run before the timed region and are reported in the same line with their own figures.
Inputs are resident (graph, shard and cache in HBM, remote rows pinned) before timing starts.

The headline workload is Large (the papers100M-shaped configuration); Mid is reported as a second
block of the same line.  The timed region is `reps` repetitions of `--steps` steps back to back
(reps * steps distinct minibatches, no synchronisation in between), so every kernel is launched
some twenty times whatever --steps is; `ms_per_step` = region / (reps * steps).

Prints ONE JSON line; see the design doc for the byte accounting behind `roofline`.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X datasheet HBM3E bandwidth
PCIE_PEAK_GBS = 64.0           # PCIe Gen5 x16, one direction

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, scaled by the
# same counters on the library's plain copy kernel over 1 GiB (`--phase calibrate`); the summaries with
# their commands are under profiles/.  Keyed by (workload, minibatches per gather launch); other shapes
# report null.
MEASURED_TRAFFIC = {
    ("large", 64): {"gather_hit": 1.385e+09, "sampler_call": 5.571e+08, "vip_dense_hop": 4.831e+10},
    ("mid", 64): {"gather_hit": 2.28e+09, "sampler_call": 7.06e+08, "vip_dense_hop": 8.44e+08},
}


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def alpha_sweep(args, cfg, spp, S, torch, ctx, G, g, Tk, p, local, remote, lo, hi):
    """Cache quality over the replication factor: VIP-ranked against degree-ranked (Sec. 3.2, Fig. 2)."""
    alphas = [0.0, 0.05, 0.1, 0.2, 0.5]
    row_bytes = cfg.D * cfg.elem_bytes
    # "deg.": in-list count (how many vertices can sample u), only for vertices reachable from the
    # partition's training set (p > 0)
    indeg = torch.bincount(g.col.long(), minlength=g.N).to(torch.float32)
    deg_score = torch.where(p > 0, indeg, torch.zeros_like(indeg))
    del indeg
    batches = [b for b in S.epoch_batches(cfg, Tk, 0) if b.numel() == min(cfg.B, Tk.numel())][:args.sweep_batches]
    bufs = spp.MFGBuffers(local.device, cfg.B, cfg.fanouts, cfg.N)
    out = torch.empty((bufs.nb[-1], cfg.D), dtype=cfg.torch_dtype, device=local.device)
    rows = []
    for policy, score in (("vip", p), ("degree", deg_score)):
        cache = spp.build_vip_cache(ctx, score, lo, hi, cfg.K, max(alphas), remote, cfg.D, cfg.elem_bytes)
        for a in alphas:
            cache.set_limit(min(cfg.cache_capacity(a), cache.n_cached))
            tot = dict(n_local=0, n_cache_hit=0, n_miss=0)
            ctx.timing(True)
            for i, seeds in enumerate(batches):
                m = spp.sample_mfg(ctx, G, seeds, cfg.fanouts, cfg.seed_sampler, i, out=bufs)
                _, st = spp.gather_features(ctx, cache, local, cfg.N, lo, hi, remote, bufs.node_ids, n=m.n[-1], out=out)
                for k in tot:
                    tot[k] += st[k]
            ms, cnt = ctx.times()
            ctx.timing(False)
            nb = len(batches)
            remote_rows = tot["n_cache_hit"] + tot["n_miss"]
            rows.append({"policy": policy, "alpha": a, "cached_rows": min(cfg.cache_capacity(a), cache.n_cached),
                         "hit_rate_of_remote": tot["n_cache_hit"] / max(remote_rows, 1),
                         "miss_rows_per_batch": tot["n_miss"] / nb,
                         "host_miss_bytes_per_batch": tot["n_miss"] * row_bytes / nb,
                         "gather_hit_ms": ms[10] / max(cnt[10], 1), "gather_miss_ms": ms[11] / max(cnt[11], 1)})
            log(rows[-1])
        cache.close()
    print(json.dumps({"phase": "alpha-sweep", "workload": cfg.name, "N": g.N, "M": g.M, "batches": len(batches),
                      "rows": rows}), flush=True)


def policy_sweep(args, cfg, spp, S, torch, ctx, G, g, Tk, p, lo, hi):
    """Remote vertices fetched per epoch (communication volume in vertices) over alpha for the caching
    policies that need nothing but the graph, the sampler and Prop. 1: none, deg., sim. (access counts
    over 2 simulated epochs), VIP (analytic), oracle (retroactive counts over the evaluated epochs) --
    the experiment shape of the policy comparison in Sec. 3.2."""
    alphas = [0.05, 0.1, 0.2, 0.5, 1.0]
    dev = p.device
    Gsz = 8
    bufs = [spp.MFGBuffers(dev, cfg.B, cfg.fanouts, cfg.N) for _ in range(Gsz)]

    def count_epochs(epochs):
        cnt = torch.zeros(cfg.N, dtype=torch.float32, device=dev)
        nb = 0
        for ep in epochs:
            batches = S.epoch_batches(cfg, Tk, ep)
            for g0 in range(0, len(batches), Gsz):
                grp = batches[g0:g0 + Gsz]
                spp.sample_mfg_multi(ctx, G, [(b, ep * 100000 + g0 + k, bufs[k]) for k, b in enumerate(grp)],
                                     cfg.fanouts, cfg.seed_sampler, sync=False)
                spp.access_count(ctx, [(bufs[k].node_ids, bufs[k].nb[-1], bufs[k].n_final_device)
                                       for k in range(len(grp))], cfg.N, cnt, sync=False)
                nb += len(grp)
        ctx.sync()
        return cnt, nb

    E = args.sweep_epochs
    t = time.time()
    sim, nb_sim = count_epochs([1000, 1001])                      # simulated epochs, disjoint from the evaluated ones
    sim_s = time.time() - t
    t = time.time()
    ev, nb_ev = count_epochs(list(range(E)))
    ev_s = time.time() - t
    log(f"sim. counts: {nb_sim} minibatches in {sim_s:.2f}s; evaluated: {nb_ev} minibatches in {ev_s:.2f}s")
    indeg = torch.bincount(g.col.long(), minlength=g.N).to(torch.float32)
    deg_score = torch.where(p > 0, indeg, torch.zeros_like(indeg))
    del indeg
    remote_mask = torch.ones(cfg.N, dtype=torch.bool, device=dev)
    remote_mask[lo:hi] = False
    total = float(ev[remote_mask].double().sum().item())
    rows = [{"policy": "none", "alpha": 0.0, "cached": 0, "remote_vertices_per_epoch": total / E}]
    for policy, score in (("deg.", deg_score), ("sim.", sim), ("VIP", p), ("oracle", ev)):
        cache = spp.build_vip_cache(ctx, score, lo, hi, cfg.K, max(alphas), None, cfg.D, cfg.elem_bytes)
        saved = torch.cumsum(ev[cache.ids.long()].double(), 0)        # accesses absorbed by the first c ranks
        for a in alphas:
            c = min(cfg.cache_capacity(a), cache.n_cached)
            kept = float(saved[c - 1].item()) if c > 0 else 0.0
            rows.append({"policy": policy, "alpha": a, "cached": c, "remote_vertices_per_epoch": (total - kept) / E})
        cache.close()
    best = {r["alpha"]: r["remote_vertices_per_epoch"] for r in rows if r["policy"] == "oracle"}
    for r in rows:
        r["vs_oracle"] = (r["remote_vertices_per_epoch"] / best[r["alpha"]]) if best.get(r["alpha"]) else None
        log(r)
    print(json.dumps({"phase": "policy-sweep", "workload": cfg.name, "N": g.N, "M": g.M, "epochs": E,
                      "minibatches": nb_ev, "sim_minibatches": nb_sim, "sim_count_s": sim_s, "rows": rows}), flush=True)


def general_phase(args, cfg, spp, S, torch, ctx, G, g, Tk, p):
    """Proposition 1 and the sampler with given transition probabilities (Sec. 3.1), timed on the
    uniform instantiation t = min(1, f_h/d(v)) so that the sizes are those of the fanout workload."""
    dev = p.device
    deg = (g.rowptr[1:] - g.rowptr[:-1])
    t = []
    for f in cfg.fanouts:
        per_row = torch.clamp(float(f) / deg.clamp(min=1).to(torch.float64), max=1.0).to(torch.float32)
        t.append(torch.repeat_interleave(per_row, deg))
    p0 = torch.zeros(cfg.N, dtype=torch.float32, device=dev)
    p0[Tk.long()] = min(1.0, cfg.B / Tk.numel())
    pg = spp.vip_propagate_general(ctx, G, p0, t, cfg.L)
    ctx.timing(True)
    for _ in range(args.vip_reps):
        pg = spp.vip_propagate_general(ctx, G, p0, t, cfg.L, sync=False)
    ms, cnt = ctx.times()
    ctx.timing(False)
    rel = ((pg - p).abs() / p.clamp(min=1e-30)).max().item()
    batches = [b for b in S.epoch_batches(cfg, Tk, 0) if b.numel() == min(cfg.B, Tk.numel())][:8]
    nb, eb = spp.mfg_bound(cfg.B, cfg.fanouts, cfg.N)
    caps = (nb[-1], [2 * e for e in eb[1:]])            # independent inclusion: sizes vary around the fanout's
    bufs = [spp.MFGBuffers(dev, 0, (), cfg.N, capacities=caps) for _ in batches]
    fb = [spp.MFGBuffers(dev, cfg.B, cfg.fanouts, cfg.N) for _ in batches]
    items = [(b, i, bufs[i]) for i, b in enumerate(batches)]
    fitems = [(b, i, fb[i]) for i, b in enumerate(batches)]
    spp.sample_mfg_general(ctx, G, t, items, cfg.L, cfg.seed_sampler)
    spp.sample_mfg_multi(ctx, G, fitems, cfg.fanouts, cfg.seed_sampler)
    res = {}
    for name, fn in (("general", lambda: spp.sample_mfg_general(ctx, G, t, items, cfg.L, cfg.seed_sampler, sync=False)),
                     ("fanout", lambda: spp.sample_mfg_multi(ctx, G, fitems, cfg.fanouts, cfg.seed_sampler, sync=False))):
        ctx.timing(True)
        for _ in range(10):
            fn()
        m2, c2 = ctx.times()
        ctx.timing(False)
        res[name] = m2[9] / max(c2[9], 1)
    print(json.dumps({"phase": "general", "workload": cfg.name, "N": g.N, "M": g.M,
                      "vip_general_ms_total": ms[0] / max(cnt[0], 1),
                      "vip_general_ms_per_hop": [ms[1 + h] / max(cnt[1 + h], 1) for h in range(cfg.L)],
                      "max_rel_diff_to_uniform_entry_point": rel,
                      "sampler_general_ms_per_8_minibatches": res["general"],
                      "sampler_fanout_ms_per_8_minibatches": res["fanout"],
                      "general_nodes_per_batch": sum(b.n[-1] for b in bufs) / len(bufs),
                      "fanout_nodes_per_batch": sum(b.n[-1] for b in fb) / len(fb)}), flush=True)


def beta_sweep(args, cfg, spp, S, torch, ctx, G, g, Tk, p, local, remote, lo, hi):
    """Host reads for local vertices over the device-resident share beta of the partition's rows:
    VIP order against the id order (Sec. 3.2 on host-to-device transfers; the experiment shape of the
    figure on local partition storage on CPU versus GPU)."""
    betas = [0.0, 0.02, 0.05, 0.1, 0.2, 0.5, 1.0]
    row_bytes = cfg.D * cfg.elem_bytes
    local_host = torch.empty(tuple(local.shape), dtype=local.dtype).pin_memory()
    local_host.copy_(local)
    cache = spp.build_vip_cache(ctx, p, lo, hi, cfg.K, cfg.alpha, remote, cfg.D, cfg.elem_bytes)
    batches = [b for b in S.epoch_batches(cfg, Tk, 0) if b.numel() == min(cfg.B, Tk.numel())][:args.sweep_batches]
    bufs = [spp.MFGBuffers(local.device, cfg.B, cfg.fanouts, cfg.N) for _ in batches]
    outs = [torch.empty((bufs[0].nb[-1], cfg.D), dtype=cfg.torch_dtype, device=local.device) for _ in batches]
    spp.sample_mfg_multi(ctx, G, [(b, i, bufs[i]) for i, b in enumerate(batches)], cfg.fanouts, cfg.seed_sampler)
    lists = [(bufs[i].node_ids, bufs[i].nb[-1], bufs[i].n_final_device, outs[i]) for i in range(len(batches))]
    rows = []
    for order, score in (("vip", p), ("id (no reorder)", torch.zeros_like(p))):
        t = time.time()
        store = spp.build_local_store(ctx, score, lo, hi, 1.0, local_host)
        build_s = time.time() - t
        for beta in betas:
            n_dev = int(beta * (hi - lo))
            store.set_limit(n_dev)
            spp.gather_features_multi(ctx, cache, store, cfg.N, lo, hi, remote, lists)          # warm-up
            ctx.timing(True)
            st = spp.gather_features_multi(ctx, cache, store, cfg.N, lo, hi, remote, lists)
            ms, cnt = ctx.times()
            ctx.timing(False)
            nb = len(batches)
            rows.append({"order": order, "beta": beta, "device_rows": n_dev, "build_s": build_s,
                         "local_rows_per_batch": st["n_local"] / nb,
                         "local_host_rows_per_batch": st["n_local_host"] / nb,
                         "local_served_from_device": 1.0 - st["n_local_host"] / max(st["n_local"], 1),
                         "local_host_bytes_per_batch": st["n_local_host"] * row_bytes / nb,
                         "remote_miss_rows_per_batch": st["n_miss"] / nb,
                         "gather_hit_ms": ms[10] / max(cnt[10], 1), "gather_miss_ms": ms[11] / max(cnt[11], 1)})
            log(rows[-1])
        store.close()
    cache.close()
    print(json.dumps({"phase": "beta-sweep", "workload": cfg.name, "N": g.N, "M": g.M, "batches": len(batches),
                      "alpha": cfg.alpha, "rows": rows}), flush=True)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.lower().startswith("model name"):
                    return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def host_threads():
    """Worker threads for the all-cores oracle leg: the machine's CPU share (16 for one GPU), at most what the process may use."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def setup_workload(args, cfg, spp, S, torch, dev, ctx, rows=True, remote_on_device=False):
    """Inputs of one workload, resident before anything is timed."""
    lo, hi = cfg.bounds()
    t = time.time()
    g = S.make_graph(cfg, dev)
    T_all = S.make_training_set(cfg, dev)
    Tk = S.local_training_set(cfg, T_all)
    del T_all
    log(f"{cfg.name}: graph N={g.N} M={g.M} |T_k|={Tk.numel()} ({time.time() - t:.1f}s)")
    t = time.time()
    G = spp.Graph(ctx, g.rowptr, g.col, in_lists=True, chunked=args.vip_layout == "chunked")
    t_inlists = time.time() - t
    nrem = cfg.N - (hi - lo)
    local = remote = None
    if rows:
        local = S.feature_block(cfg, lo, hi, dev)
        if remote_on_device:
            remote = torch.empty((nrem, cfg.D), dtype=cfg.torch_dtype, device=dev)
        else:
            remote = torch.empty((nrem, cfg.D), dtype=cfg.torch_dtype).pin_memory()
        for a in range(0, nrem, 1 << 19):
            b = min(nrem, a + (1 << 19))
            remote[a:b].copy_(S.feature_rows(cfg, S.remote_ids(cfg, a, b, dev)))
        torch.cuda.synchronize()
        log(f"{cfg.name}: features local {tuple(local.shape)} remote {tuple(remote.shape)} "
            f"{'pinned' if remote.is_pinned() else 'in device memory'}; transposed structure built in {t_inlists:.2f}s")
    else:
        log(f"{cfg.name}: no feature rows for phase {args.phase}; transposed structure built in {t_inlists:.2f}s")
    return dict(g=g, Tk=Tk, G=G, t_inlists=t_inlists, local=local, remote=remote, lo=lo, hi=hi, nrem=nrem)


def time_vip(args, cfg, spp, ctx, w, group):
    """Proposition 1 on the workload, timed over args.vip_reps propagations (events on the context's stream)."""
    g, G, Tk = w["g"], w["G"], w["Tk"]
    p = spp.vip_propagate(ctx, G, Tk, cfg.B, cfg.fanouts)            # warm-up, allocates workspaces
    ctx.timing(True)
    for _ in range(args.vip_reps):
        p = spp.vip_propagate(ctx, G, Tk, cfg.B, cfg.fanouts, sync=False)
    ms, cnt, mn, med = ctx.time_stats()
    ctx.timing(False)
    total_ms = ms[0] / max(cnt[0], 1)
    hop_ms = [ms[1 + h] / max(cnt[1 + h], 1) for h in range(cfg.L)]
    hop_med = [med[1 + h] for h in range(cfg.L)]
    hop_min = [mn[1 + h] for h in range(cfg.L)]
    # algorithmic bytes of one hop (independent of how the transposed edges are laid out): one int32
    # source id per edge, one 64-bit offset per destination row, y read once, the per-vertex result
    # written once
    hop_bytes = 4 * g.M + 8 * (g.N + 1) + 4 * g.N + 4 * g.N
    pushed, frontier_edges = spp.vip_last_hops(ctx, cfg.L)
    dense = [h for h in range(cfg.L) if not pushed[h]]               # only a pulled hop streams all M edges
    roof = None
    if dense:
        h = max(dense, key=lambda i: hop_ms[i])
        roof = {"bound": "hbm", "achieved": hop_bytes / (hop_ms[h] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "kernel": "dense hop of spp_vip_propagate (slowest hop that walks all M edges), all its launches",
                "hop": h + 1, "avg_launch_ms": hop_ms[h], "median_launch_ms": hop_med[h], "min_launch_ms": hop_min[h],
                "launches": cnt[1 + h], "bytes_per_launch": hop_bytes,
                "traffic": MEASURED_TRAFFIC.get((cfg.name, group), {}).get("vip_dense_hop")}
        roof["frac"] = roof["achieved"] / HBM_PEAK_GBS
    block = {"ms_total": total_ms, "ms_per_hop": hop_ms, "bytes_per_hop": hop_bytes, "roofline": roof,
             "hop_pushed_over_sparse_frontier": pushed, "frontier_out_edges_per_hop": frontier_edges,
             "propagations_timed": cnt[0], "in_lists_build_s": w["t_inlists"]}
    return p, block


def cpu_legs(args, cfg, spp, S, torch, np, ctx, w, cache, batches, first, count, p):
    """The oracle as it stands on the machine's host cores: one thread, then the same single-thread code
    with minibatches spread over threads (the C calls release the interpreter lock); once each the
    oracle's VIP propagation and cache ranking (set-up rows)."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    g, lo, hi, local, remote = w["g"], w["lo"], w["hi"], w["local"], w["remote"]
    rp, col = g.rowptr.cpu().numpy(), g.col.cpu().numpy()
    as_np = (lambda t: t.view(torch.int16).numpy()) if cfg.dtype == "bf16" else (lambda t: t.numpy())
    local_np = as_np(local.cpu())
    remote_np = as_np(remote)
    ids_np = cache.ids.cpu().numpy()
    crow_np = as_np(S.feature_rows(cfg, cache.ids.long()).cpu())
    seeds_np = {}

    def one(i):
        if i not in seeds_np:
            seeds_np[i] = batches[i].cpu().numpy()
        ref = oracle.sample_mfg(rp, col, seeds_np[i], cfg.fanouts, cfg.seed_sampler, i)
        oracle.gather(cfg.N, lo, hi, local_np, crow_np, ids_np, remote_np, ref.node_ids)
        return None                      # the rows are not kept: thousands of minibatches pass through here

    for i in range(first, first + count):
        seeds_np[i] = batches[i].cpu().numpy()
    budget = args.cpu_seconds
    # one thread
    nb, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < budget and nb < 50 * count:
        one(first + nb % count)
        nb += 1
    spent1 = time.perf_counter() - t0
    single = {"value": nb / spent1, "unit": "minibatches/s", "cores": 1,
              "sample": f"{nb} of the timed minibatches (sample_mfg + gather), {spent1:.1f}s"}
    # all cores: the same calls, minibatches dealt to threads
    C = host_threads()
    per = max(1, int(nb / max(spent1, 1e-9) * budget))              # what one thread gets through in the budget
    todo = [first + k % count for k in range(per * C)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=C) as ex:
        for _ in ex.map(one, todo):
            pass
    spentC = time.perf_counter() - t0
    cpu = {"value": len(todo) / spentC, "unit": "minibatches/s", "cores": C, "kind": "oracle",
           "sample": f"{len(todo)} minibatches drawn from the {count} first timed ones (sample_mfg + gather each), dealt to "
                     f"{C} threads running the single-thread oracle, {spentC:.1f}s of wall time",
           "cpu_model": cpu_model(), "host_cpus_visible": os.cpu_count(), "one_thread": single}
    if args.cpu_setup == "on":
        Tk_np = w["Tk"].cpu().numpy()
        t0 = time.perf_counter()
        p_ref, _ = oracle.vip(rp, col, Tk_np, cfg.B, cfg.fanouts)
        vip_s = time.perf_counter() - t0
        err = np.abs(p.cpu().numpy().astype(np.float64) - p_ref)
        vip_ok = bool(np.all(err <= 1e-5 * p_ref + 1e-37))
        p_np = p.cpu().numpy()
        t0 = time.perf_counter()
        ids_ref = oracle.cache_select(p_np, lo, hi, cfg.K, cfg.alpha)
        sel_s = time.perf_counter() - t0
        sel_ok = bool(np.array_equal(ids_ref, ids_np))
        if not (vip_ok and sel_ok):
            log(f"PARITY FAILURE against the oracle: vip ok={vip_ok}, cache ids ok={sel_ok}")
            sys.exit(1)
        cpu["setup_rows_one_thread"] = {"vip_propagate_s": vip_s, "cache_select_s": sel_s,
                                        "checked_against_hip_path": "all N probabilities to 1e-5 relative, all cache ids bit-exact"}
    return cpu, (rp, col, local_np, remote_np, ids_np, crow_np)


def run_workload(args, cfg, spp, S, torch, np, dev, K, W, R, cpu_leg):
    """All figures of one workload: set-up rows (VIP, cache), the timed pipeline, roofline, PCIe, CPU legs."""
    P = max(1, args.pipeline)
    total_steps = K * R
    Gsz = max(1, min(args.group, 64, -(-total_steps // P)))
    row_bytes = cfg.D * cfg.elem_bytes
    ctx = spp.Context(0)
    w = setup_workload(args, cfg, spp, S, torch, dev, ctx)
    g, G, Tk, local, remote, lo, hi, nrem = (w[k] for k in ("g", "G", "Tk", "local", "remote", "lo", "hi", "nrem"))

    # ---- one-time rows: VIP propagation, cache ranking + fill -------------------------------
    p, vip = time_vip(args, cfg, spp, ctx, w, Gsz)
    t = time.time()
    cache = spp.build_vip_cache(ctx, p, lo, hi, cfg.K, cfg.alpha, remote, cfg.D, cfg.elem_bytes)
    torch.cuda.synchronize()
    cache_s = time.time() - t
    vip["cache_build_s"] = cache_s
    vip["n_cached"] = cache.n_cached
    log(f"{cfg.name}: vip {vip['ms_total']:.3f} ms (hops {['%.3f' % x for x in vip['ms_per_hop']]}), "
        f"cache {cache.n_cached} rows in {cache_s:.3f}s")

    # ---- minibatches -------------------------------------------------------------------------
    batches = []
    ep = 0
    while len(batches) < W + total_steps:
        batches.extend(b for b in S.epoch_batches(cfg, Tk, ep) if b.numel() == min(cfg.B, Tk.numel()))
        ep += 1
    batches = batches[:W + total_steps]
    # A lane = one context (stream, side stream, workspaces) with two sets of `group` MFG buffers and
    # output rows, used alternately.  Per group the lane samples `group` minibatches with one call,
    # then gathers all of them with one classification, one hit copy and one miss copy.  The miss
    # copy is left running on the side stream (SPP_NO_JOIN) while the lane samples the next group
    # into its other buffer set; the stream joins it (where a consumer of the rows would sit) just
    # before the next hit copy.
    lanes = []
    for k in range(P):
        c = ctx if k == 0 else spp.Context(0, stream=torch.cuda.Stream(dev))
        sets = []
        for _ in range(2):
            b = [spp.MFGBuffers(dev, cfg.B, cfg.fanouts, cfg.N) for _ in range(Gsz)]
            o = [torch.empty((b[0].nb[-1], cfg.D), dtype=cfg.torch_dtype, device=dev) for _ in range(Gsz)]
            sets.append((b, o))
        lanes.append((c, sets))
    state = {"store_order": args.store_order == "on"}

    def run(first, count, gsz=None, order=None, gi0=0, beside=False):
        """Enqueue minibatches first .. first+count-1 (no host synchronisation inside)."""
        gsz = Gsz if gsz is None else gsz
        order = state["store_order"] if order is None else order
        gi = gi0
        for g0 in range(first, first + count, gsz):
            c, sets = lanes[gi % P]
            b, o = sets[(gi // P) % 2]
            gi += 1
            idx = range(g0, min(g0 + gsz, first + count))
            spp.sample_mfg_multi(c, G, [(batches[i], i, b[k]) for k, i in enumerate(idx)], cfg.fanouts,
                                 cfg.seed_sampler, sync=False)
            # the gather classifies this group beside the previous group's miss copy, waits for that
            # copy (the previous group's rows are complete from there on), then copies the hits
            spp.gather_features_multi(c, cache, local, cfg.N, lo, hi, remote,
                                      [(b[k].node_ids, b[k].nb[-1], b[k].n_final_device, o[k]) for k in range(len(idx))],
                                      sync=False, join=False, store_order=order, hit_beside_miss=beside)
        for c, _ in lanes:
            spp.gather_join(c)

    # set-up, not a step: every lane runs two full groups once, so that both buffer sets and both sets of
    # library workspaces exist before the warm-up (an allocation inside the timed region would stall it)
    torch.cuda.synchronize()
    for c, _ in lanes:
        c.totals(reset=True)
    n_setup = min(len(batches), 2 * P * Gsz)
    run(0, n_setup)
    torch.cuda.synchronize()
    # share of the remote store's rows that one group fetches: decides the order of the fetches
    fetched = sum(t_["n_miss"] - t_["n_miss_shared"] for t_ in (c.totals(reset=True) for c, _ in lanes))
    fetched_share = fetched / max(1, -(-n_setup // Gsz)) / max(nrem, 1)
    if args.store_order == "auto":
        state["store_order"] = fetched_share >= 0.125
    log(f"{cfg.name}: a group fetches {fetched_share:.3f} of the remote store's rows; store order: {state['store_order']}")
    if W > 0:
        run(0, W)
    torch.cuda.synchronize()
    for c, _ in lanes:
        c.timing(True)
        c.totals(reset=True)
    torch.cuda.synchronize()
    # the timed region: R repetitions of K steps back to back (R*K distinct minibatches), no
    # synchronisation in between, so that the miss copy of a group overlaps the sampling of the next
    t0 = time.perf_counter()
    run(W, total_steps)
    for c, _ in lanes:
        c.sync()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms, cnt, shortest, median = [0.0] * 16, [0] * 16, [0.0] * 16, [0.0] * 16
    for li, (c, _) in enumerate(lanes):
        m_, c_, mn_, med_ = c.time_stats()
        ms = [a + b for a, b in zip(ms, m_)]
        cnt = [a + b for a, b in zip(cnt, c_)]
        if li == 0:
            shortest, median = mn_, med_           # of the first lane's launches
        c.timing(False)
    elapsed = t1 - t0

    # per-batch averages from the contexts' device-side running sums (no extra pass, no host sync)
    tot = dict(n_nodes=0, n_edges=0, n_local=0, n_cache_hit=0, n_miss=0, n_miss_shared=0)
    for c, _ in lanes:
        t_ = c.totals()
        for k in tot:
            tot[k] += t_[k]
    avg = {k: v / total_steps for k, v in tot.items()}

    # the same steps at the pipeline depth the paper keeps (ten minibatches in flight: groups of five on
    # the two buffer sets), for comparison: reported beside `value`, never as it
    depth = None
    if args.depth_leg == "on" and P == 1 and Gsz > 5 and total_steps >= 40:
        kd = min(total_steps, 320) // 5 * 5
        run(W, 20, gsz=5, order=False)
        torch.cuda.synchronize()
        td = time.perf_counter()
        run(W, kd, gsz=5, order=False)
        for c, _ in lanes:
            c.sync()
        torch.cuda.synchronize()
        td = time.perf_counter() - td
        depth = {"minibatches_per_gather_launch": 5, "minibatches_in_flight": 10, "steps": kd,
                 "value": kd / td, "ms_per_step": td / kd * 1e3}

    # the same steps with each group's miss copy queued BEFORE its hit copy (SPP_HIT_BESIDE_MISS): the link never
    # idles, the hit copy shares the chip with a miss copy.  Reported beside `value`, never as it: the headline keeps
    # the HBM-bound kernel at its full rate.
    beside = None
    if args.depth_leg == "on" and P == 1:
        run(W, min(W, total_steps) or Gsz, beside=True)
        torch.cuda.synchronize()
        ctx.timing(True)
        tb = time.perf_counter()
        run(W, total_steps, beside=True)
        ctx.sync()
        torch.cuda.synchronize()
        tb = time.perf_counter() - tb
        mb_, cb_, _, medb_ = ctx.time_stats()
        ctx.timing(False)
        hb = mb_[10] / max(cb_[10], 1)
        beside = {"order": "miss copy of a group queued before its hit copy (SPP_HIT_BESIDE_MISS)",
                  "value": total_steps / tb, "ms_per_step": tb / total_steps * 1e3, "steps": total_steps,
                  "gather_hit_avg_launch_ms": hb, "gather_hit_median_launch_ms": medb_[10], "launches": cb_[10]}

    # the hit copy by itself, for comparison: as many rows as a timed launch copies, drawn at random from the local
    # shard, one list, nothing else on the chip.  Reported beside the pipeline's figure, never as it.
    alone = None
    if args.depth_leg == "on" and P == 1:
        n_alone = int((tot["n_local"] + tot["n_cache_hit"]) / max(cnt[10], 1))
        if n_alone > 0:
            gen = torch.Generator(device=dev)
            gen.manual_seed(77)
            # other rows at every launch: the caches must not hold what the launch before read
            ids_alone = [(torch.randint(0, hi - lo, (n_alone,), device=dev, generator=gen, dtype=torch.int64) + lo).to(torch.int32)
                         for _ in range(11)]
            out_alone = torch.empty((n_alone, cfg.D), dtype=cfg.torch_dtype, device=dev)
            spp.gather_features(ctx, None, local, cfg.N, lo, hi, None, ids_alone[10], out=out_alone)
            ctx.timing(True)
            for k in range(10):
                spp.gather_features(ctx, None, local, cfg.N, lo, hi, None, ids_alone[k], out=out_alone, sync=False)
            ctx.sync()
            ma_, ca_, _, meda_ = ctx.time_stats()
            ctx.timing(False)
            ha = ma_[10] / max(ca_[10], 1)
            alone = {"rows": n_alone, "avg_launch_ms": ha, "median_launch_ms": meda_[10], "launches": ca_[10],
                     "frac": n_alone * 2 * row_bytes / (ha * 1e-3) / 1e9 / HBM_PEAK_GBS if ha > 0 else None,
                     "what": "the same kernel on one list of as many random rows of the local shard (other rows at every launch), alone on the chip"}
            del ids_alone, out_alone

    T_HIT, T_MISS, T_CLS, T_SAMPLE = 10, 11, 12, 9
    per = lambda i: ms[i] / max(cnt[i], 1)
    hit_ms, miss_ms, cls_ms, sample_ms = per(T_HIT), per(T_MISS), per(T_CLS), per(T_SAMPLE)
    # per LAUNCH: a launch of the hit / miss kernel covers one group of minibatches
    n_launch = max(cnt[T_HIT], 1)
    hit_rows = (tot["n_local"] + tot["n_cache_hit"]) / n_launch
    hit_bytes = hit_rows * 2 * row_bytes                 # read the source row + write the output row
    roof = {"bound": "hbm", "achieved": hit_bytes / (hit_ms * 1e-3) / 1e9 if hit_ms > 0 else 0.0,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "kernel": "gather_hit_kernel<16>",
            "traffic": MEASURED_TRAFFIC.get((cfg.name, Gsz), {}).get("gather_hit") if P == 1 else None,
            "bytes_per_launch": hit_bytes, "rows_per_launch": hit_rows, "avg_launch_ms": hit_ms,
            "median_launch_ms": median[T_HIT], "min_launch_ms": shortest[T_HIT], "launches": cnt[T_HIT],
            "note": "runs between two PCIe miss copies, with the whole chip", "same_kernel_alone": alone}
    roof["frac"] = roof["achieved"] / HBM_PEAK_GBS
    if beside is not None and beside["gather_hit_avg_launch_ms"] > 0:
        beside["gather_hit_frac_of_hbm_peak"] = hit_bytes / (beside["gather_hit_avg_launch_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS
    # bytes that cross PCIe: a vertex missed by several minibatches of a group is read once and copied on the device
    miss_bytes = (tot["n_miss"] - tot["n_miss_shared"]) / max(cnt[T_MISS], 1) * row_bytes
    pcie = {"bound": "pcie", "achieved": miss_bytes / (miss_ms * 1e-3) / 1e9 if miss_ms > 0 else 0.0,
            "peak": PCIE_PEAK_GBS, "unit": "GB/s", "kernel": "gather_miss_kernel<16> (side stream)",
            "bytes_per_launch": miss_bytes, "avg_launch_ms": miss_ms, "launches": cnt[T_MISS],
            "rows_missed_per_launch": tot["n_miss"] / max(cnt[T_MISS], 1),
            "rows_shared_per_launch": tot["n_miss_shared"] / max(cnt[T_MISS], 1)}
    pcie["frac"] = pcie["achieved"] / PCIE_PEAK_GBS
    # the sampler has no %-of-peak bar (latency and transaction bound): algorithmic bytes as context
    sample_bytes = (16 * tot["n_edges"] + 20 * (tot["n_nodes"])) / max(cnt[T_SAMPLE], 1)
    sampler = {"avg_call_ms": sample_ms, "median_call_ms": median[T_SAMPLE], "min_call_ms": shortest[T_SAMPLE],
               "calls": cnt[T_SAMPLE], "minibatches_per_call": Gsz, "algorithmic_bytes_per_call": sample_bytes,
               "algorithmic_GBps": sample_bytes / (sample_ms * 1e-3) / 1e9 if sample_ms > 0 else 0.0,
               "traffic": MEASURED_TRAFFIC.get((cfg.name, Gsz), {}).get("sampler_call")}

    # ---- the launch configuration that was timed, checked against the oracle ------------------
    cpu = None
    checked = []
    if cpu_leg and args.cpu_seconds > 0:
        cpu, host = cpu_legs(args, cfg, spp, S, torch, np, ctx, w, cache, batches, W, min(total_steps, 256), p)
        import oracle
        rp, col, local_np, remote_np, ids_np, crow_np = host
        # one more group through the timed calls (same group size, flags and deferred join); its first three
        # minibatches and one drawn at random are compared with the oracle
        c, sets = lanes[0]
        b, o = sets[0]
        idx = list(range(W, W + min(Gsz, total_steps)))
        run(W, len(idx))
        c.sync()
        torch.cuda.synchronize()
        rng = np.random.default_rng(12345)
        pick = sorted(set(list(range(min(3, len(idx)))) + ([int(rng.integers(3, len(idx)))] if len(idx) > 3 else [])))
        for k in pick:
            i = idx[k]
            ref = oracle.sample_mfg(rp, col, batches[i].cpu().numpy(), cfg.fanouts, cfg.seed_sampler, i)
            want, _, counts = oracle.gather(cfg.N, lo, hi, local_np, crow_np, ids_np, remote_np, ref.node_ids)
            cn = b[k].counts.cpu().numpy()
            n_h = [int(x) for x in cn[:cfg.L + 1]]
            e_h = [int(x) for x in cn[9:9 + cfg.L + 1]]
            got = o[k][:n_h[-1]]
            got = (got.view(torch.int16) if cfg.dtype == "bf16" else got).cpu().numpy()
            ok = (n_h == ref.n and e_h == ref.e
                  and np.array_equal(b[k].node_ids[:n_h[-1]].cpu().numpy(), ref.node_ids)
                  and all(np.array_equal(b[k].indptr[h][:n_h[h] + 1].cpu().numpy(), ref.indptr[h]) for h in range(cfg.L))
                  and all(np.array_equal(b[k].src[h][:e_h[h + 1]].cpu().numpy(), ref.src[h]) for h in range(cfg.L))
                  and np.array_equal(got.view(np.uint8), want.view(np.uint8)))
            if not ok:
                log(f"PARITY FAILURE against the oracle on minibatch {i} of {cfg.name}")
                sys.exit(1)
            checked.append(i)
        cpu["checked_against_hip_path"] = (f"minibatches {checked} of a group of {len(idx)} run through the timed calls "
                                           "(MFGs, relabel maps and gathered rows bit-exact)")
        del rp, col, local_np, remote_np, ids_np, crow_np, host

    block = {
        "value": total_steps / elapsed, "unit": "minibatches/s", "ms_per_step": elapsed / total_steps * 1e3,
        "timed_region_s": elapsed,
        "dtype": {"fp32": "f32", "fp16": "f16", "bf16": "bf16"}[cfg.dtype] + " rows (byte copy), int32 ids",
        "config": {"workload": f"{cfg.name}: N={g.N} M={g.M} D={cfg.D} {cfg.dtype} fanouts={list(cfg.fanouts)} "
                               f"B={cfg.B} K={cfg.K} alpha={cfg.alpha} owned partition {cfg.owned_partition}",
                   "reps": R, "steps_timed": total_steps,
                   "lanes": P, "minibatches_per_gather_launch": Gsz, "minibatches_in_flight": 2 * P * Gsz,
                   "setup_minibatches_before_warmup": n_setup,
                   "at_ten_minibatches_in_flight": depth,
                   "with_hit_copy_beside_miss_copy": beside,
                   "misses_fetched_in": "store order" if state["store_order"] else "list order",
                   "share_of_remote_store_fetched_per_launch": round(fetched_share, 4),
                   "avg_per_batch": {k: round(v, 1) for k, v in avg.items()},
                   "hit_rate_of_remote": avg["n_cache_hit"] / max(avg["n_cache_hit"] + avg["n_miss"], 1e-9),
                   "features": "sum of twelve hashed 16-bit uniforms, centred, unit variance (stand-in for N(0,1); the path copies bytes)"},
        "roofline": roof, "cpu_baseline": cpu, "pcie": pcie, "sampler": sampler,
        # the overlapped pipeline against its pieces run one after the other (Sec. 4.3: what the overlap buys)
        "overlap": {"serial_sum_ms_per_step": (sample_ms + cls_ms + hit_ms + miss_ms) / max(Gsz, 1),
                    "pipelined_ms_per_step": elapsed / total_steps * 1e3,
                    "gain": (sample_ms + cls_ms + hit_ms + miss_ms) / max(Gsz, 1) / (elapsed / total_steps * 1e3)},
        "kernels_ms": {"sample_mfg_per_launch": sample_ms, "gather_classify_per_launch": cls_ms,
                       "gather_hit_per_launch": hit_ms, "gather_miss_per_launch": miss_ms,
                       "median": {"sample_mfg": median[T_SAMPLE], "gather_classify": median[T_CLS],
                                  "gather_hit": median[T_HIT], "gather_miss": median[T_MISS]},
                       "min": {"sample_mfg": shortest[T_SAMPLE], "gather_classify": shortest[T_CLS],
                               "gather_hit": shortest[T_HIT], "gather_miss": shortest[T_MISS]}},
        "vip": vip,
    }
    cache.close()
    G.close()
    for c, _ in lanes:
        c.close()
    return block


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1280)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--reps", type=int, default=0,
                    help="the timed region is `reps` repetitions of `steps` steps back to back (reps*steps distinct minibatches, "
                         "no synchronisation in between); 0 = as many as bring the region to 1280 steps, so that every kernel "
                         "is launched 20 times whatever --steps is")
    ap.add_argument("--config", default="large",
                    help="headline workload: large (default: the papers100M-shaped configuration, the largest that the "
                         "metric's single-GPU pipeline is quoted on) | mid | tiny | wide | skew")
    ap.add_argument("--second", default="auto",
                    help="a second workload reported as a block of the same JSON line (auto: mid beside large; none)")
    ap.add_argument("--vip-reps", type=int, default=10)
    ap.add_argument("--vip-layout", default="auto", choices=["auto", "chunked"],
                    help="transposed edges: auto = row blocks up to 2^23 vertices, the chunked two-pass layout above; "
                         "chunked = the chunked layout whatever the size")
    ap.add_argument("--pipeline", type=int, default=1,
                    help="lanes: contexts (each with its own stream and buffers) used round-robin")
    ap.add_argument("--group", type=int, default=64,
                    help="minibatches a lane samples with one call and then gathers with ONE set of launches "
                         "(2 x pipeline x group minibatches are in flight; the paper keeps ten)")
    ap.add_argument("--store-order", default="auto", choices=["auto", "on", "off"],
                    help="fetch a group's missed rows in the order of the remote store (SPP_STORE_ORDER); auto: when "
                         "the set-up groups fetched an eighth or more of the store's rows per group")
    ap.add_argument("--depth-leg", default="on", choices=["on", "off"],
                    help="after the timed steps, also time the pipeline at ten minibatches in flight (the paper's depth); "
                         "off keeps a kernel trace of the run to the launches of the timed configuration")
    ap.add_argument("--cpu-seconds", type=float, default=8.0,
                    help="budget of each of the two oracle legs over minibatches (one thread, all threads); 0 = no CPU legs")
    ap.add_argument("--cpu-setup", default="on", choices=["on", "off"],
                    help="also time the oracle's VIP propagation and cache ranking once (one thread; about a minute on large)")
    ap.add_argument("--phase", default="all", choices=["all", "vip", "alpha-sweep", "beta-sweep", "policy-sweep", "general", "calibrate"],
                    help="all: the benchmark line; vip: set-up and VIP propagation only (for profiling that kernel); "
                         "alpha-sweep: hit rate and host-miss bytes per batch over alpha in {0,.05,.1,.2,.5}, VIP-ranked "
                         "against degree-ranked cache (the experiment shape of Fig. 2 / Fig. 7), e.g. with --config skew; "
                         "policy-sweep: remote vertices fetched per epoch over alpha for the policies none / deg. / sim. / "
                         "VIP / oracle (the policy comparison of Sec. 3.2), counted on the device over --sweep-epochs epochs; "
                         "general: Prop. 1 and the sampler with given transition probabilities, timed on the uniform "
                         "instantiation next to the fanout entry points; "
                         "beta-sweep: local rows read from host memory over the device-resident share beta of the "
                         "partition's rows, VIP order against id order (the experiment shape of the figure on local "
                         "storage on CPU versus GPU); "
                         "calibrate: the library's plain streaming kernels over 1 GiB (read-only, copy, write-only): the "
                         "known-size kernels that scale the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc")
    ap.add_argument("--sweep-batches", type=int, default=8)
    ap.add_argument("--sweep-epochs", type=int, default=4)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one partition's share of the method); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2305_03152_amd as spp
    from workloads import synth as S

    cfg = S.CONFIGS[args.config]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)

    def stream_rates():
        c = spp.Context(0)
        r = spp.stream_rates(c, 1 << 30, reps=10)
        c.close()
        return r

    if args.phase == "calibrate":
        r = stream_rates()
        print(json.dumps({"phase": "calibrate", "bytes_per_pass": 1 << 30, "passes": 10,
                          "kernels": "spp_stream_rates: read-only pass, copy (1 GiB read + 1 GiB written), write-only fill",
                          "GBps": r}), flush=True)
        return

    if args.phase != "all":
        ctx = spp.Context(0)
        rows = args.phase in ("alpha-sweep", "beta-sweep")
        # the beta sweep measures host reads of LOCAL rows: its remote store sits in device memory so that
        # the host's pinning limit is left to the partition's own rows
        w = setup_workload(args, cfg, spp, S, torch, dev, ctx, rows=rows, remote_on_device=args.phase == "beta-sweep")
        g, G, Tk, local, remote, lo, hi = (w[k] for k in ("g", "G", "Tk", "local", "remote", "lo", "hi"))
        p, vip = time_vip(args, cfg, spp, ctx, w, args.group)
        if args.phase == "vip":
            print(json.dumps({"phase": "vip", "workload": cfg.name, "N": g.N, "M": g.M, **vip}), flush=True)
        elif args.phase == "alpha-sweep":
            alpha_sweep(args, cfg, spp, S, torch, ctx, G, g, Tk, p, local, remote, lo, hi)
        elif args.phase == "beta-sweep":
            beta_sweep(args, cfg, spp, S, torch, ctx, G, g, Tk, p, local, remote, lo, hi)
        elif args.phase == "policy-sweep":
            policy_sweep(args, cfg, spp, S, torch, ctx, G, g, Tk, p, lo, hi)
        elif args.phase == "general":
            general_phase(args, cfg, spp, S, torch, ctx, G, g, Tk, p)
        return

    K, W = args.steps, args.warmup
    R = args.reps if args.reps > 0 else max(1, -(-1280 // max(K, 1)))
    rates = stream_rates()
    head = run_workload(args, cfg, spp, S, torch, np, dev, K, W, R, cpu_leg=True)
    second_name = {"auto": "mid" if cfg.name == "large" else "none"}.get(args.second, args.second)
    second = None
    if second_name != "none" and second_name != cfg.name:
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        try:
            torch._C._host_emptyCache()          # give the pinned remote store back before the next one is pinned
        except Exception:
            pass
        second = run_workload(args, S.CONFIGS[second_name], spp, S, torch, np, dev, K, W, R, cpu_leg=True)

    line = {
        "metric": "sampled+gathered minibatches/s per partition on 1 GPU",
        "value": head["value"], "unit": head["unit"], "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": head["config"], "roofline": head["roofline"], "cpu_baseline": head["cpu_baseline"],
        "pcie": head["pcie"], "sampler": head["sampler"], "overlap": head["overlap"], "kernels_ms": head["kernels_ms"],
        "vip": head["vip"],
        "timed_region_s": head["timed_region_s"],
        "hbm_measured": {"datasheet_peak_GBps": HBM_PEAK_GBS, "library_streaming_kernels_over_1GiB_GBps": rates,
                         "note": "the datasheet peak counts reads and writes together; achieved figures are read against it"},
    }
    if second is not None:
        line[second_name] = second
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
