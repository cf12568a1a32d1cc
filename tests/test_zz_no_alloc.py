"""The gather entry point that allocates nothing (spp_gather_features_static) against the ordinary one
(spp_gather_features), through the C interface: same rows bit for bit and same statistics on two calls
in a row, the second with a smaller input; the limit on n; device memory untouched by the calls."""
import numpy as np
import pytest
import torch

from workloads import synth as S

pytestmark = pytest.mark.gpu


def _bytes(t):
    return t.contiguous().view(torch.uint8).cpu().numpy()


def test_static_gather_matches_the_ordinary_gather():
    import paper_2305_03152_amd as spp
    spp.load_library()
    cfg = S.scaled(S.MID, 150_000)
    dev = torch.device("cuda:0")
    lo, hi = cfg.bounds()
    N = cfg.N
    ctx = spp.Context(0)
    local = S.feature_block(cfg, lo, hi, dev)
    nrem = N - (hi - lo)
    remote = torch.empty((nrem, cfg.D), dtype=cfg.torch_dtype).pin_memory()
    remote.copy_(S.feature_rows(cfg, S.remote_ids(cfg, 0, nrem, dev)))
    # a cache over a made-up score: every third remote vertex scores, so local, cached and missed ids all occur
    score = torch.zeros(N, dtype=torch.float32, device=dev)
    score[torch.arange(0, N, 3, device=dev)] = torch.rand(len(range(0, N, 3)), device=dev, generator=torch.Generator(dev).manual_seed(5)) + 0.1
    cache = spp.build_vip_cache(ctx, score, lo, hi, cfg.K, 0.5, remote, cfg.D, cfg.elem_bytes)
    gen = torch.Generator().manual_seed(3)
    first = torch.randint(0, N, (100_000,), generator=gen, dtype=torch.int32)       # several chunks, a ragged tail, duplicates
    second = torch.randint(0, N, (4_321,), generator=gen, dtype=torch.int32)        # smaller: the workspace keeps the first call's lists
    out_a = torch.empty((first.numel(), cfg.D), dtype=cfg.torch_dtype, device=dev)
    out_b = torch.empty_like(out_a)
    torch.cuda.synchronize()
    for k, ids in enumerate((first, second)):
        ids_d = ids.to(dev)
        n = ids.numel()
        out_a.fill_(-1.0)
        out_b.fill_(-2.0)
        _, st_ref = spp.gather_features(ctx, cache, local, N, lo, hi, remote, ids_d, out=out_a)
        free0 = torch.cuda.mem_get_info(0)[0]
        st = spp.gather_features_static(ctx, cache, local, N, lo, hi, remote, ids_d, out_b)
        free1 = torch.cuda.mem_get_info(0)[0]
        assert st == st_ref, (k, st, st_ref)
        assert st["n_local"] > 0 and st["n_cache_hit"] > 0 and st["n_miss"] > 0
        assert np.array_equal(_bytes(out_b[:n]), _bytes(out_a[:n])), f"call {k}"
        assert np.array_equal(_bytes(out_b[:n]), _bytes(S.feature_rows(cfg, ids_d))), f"call {k}: rows by regeneration"
        assert np.all(_bytes(out_b[n:]) == _bytes(torch.full_like(out_b[n:], -2.0))), "rows beyond n were written"
        assert free1 == free0, "device memory changed hands during the allocation-free call"
    # device-side count below the bound n, as after a sampling call
    n_dev = torch.tensor([1234], dtype=torch.int64, device=dev)
    out_b.fill_(-2.0)
    spp.gather_features_static(ctx, cache, local, N, lo, hi, remote, first.to(dev), out_b, n_device=n_dev)
    assert np.array_equal(_bytes(out_b[:1234]), _bytes(S.feature_rows(cfg, first[:1234].to(dev))))
    assert np.all(_bytes(out_b[1234:]) == _bytes(torch.full_like(out_b[1234:], -2.0)))
    # beyond the limit: an error before any work
    big = torch.zeros(spp.api.SPP_STATIC_GATHER_MAX_ROWS + 1, dtype=torch.int32, device=dev)
    big_out = torch.empty((big.numel(), cfg.D), dtype=cfg.torch_dtype, device=dev)
    with pytest.raises(spp.SppError, match="SPP_STATIC_GATHER_MAX_ROWS"):
        spp.gather_features_static(ctx, cache, local, N, lo, hi, remote, big, big_out)
    # the ordinary call still works afterwards, and so does the static one at exactly the limit
    at_limit = torch.randint(0, N, (spp.api.SPP_STATIC_GATHER_MAX_ROWS,), generator=gen, dtype=torch.int32).to(dev)
    st = spp.gather_features_static(ctx, cache, local, N, lo, hi, remote, at_limit, big_out)
    _, st_ref = spp.gather_features(ctx, cache, local, N, lo, hi, remote, at_limit, out=torch.empty_like(big_out))
    assert st == st_ref
    assert np.array_equal(_bytes(big_out[:at_limit.numel()]), _bytes(S.feature_rows(cfg, at_limit)))
    cache.close()
    ctx.close()
