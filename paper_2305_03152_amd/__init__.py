"""MI355X-native per-partition data path of VIP-cached, partitioned GNN minibatch preparation.

Four calls, each a thin binding over the C interface in include/spp.h whose work runs in
hand-written HIP kernels for gfx950: vip_propagate, build_vip_cache, sample_mfg,
gather_features.
"""
from .api import (access_count, Cache, Context, Graph, LocalStore, MFGBuffers, SppError, build_local_store, build_vip_cache, gather_features, gather_features_multi, gather_features_static, gather_join,  # noqa: F401
                  gather_last_stats, load_library, mfg_bound, stream_rates, sample_mfg, sample_mfg_general, sample_mfg_multi, vip_propagate_general, vip_propagate, vip_last_hops, EXPORTS, LIB_PATH)
