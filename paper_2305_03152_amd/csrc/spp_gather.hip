// Cache-aware feature gather (Secs. 4.1-4.3; stages 5-10 of the pipeline walkthrough in Appendix D).
//
//   classify  (main stream)  per id: range test against [lo,hi) (constant memory, Sec. 4.1), else a
//                            probe of the cache's id table (Sec. 4.2), else a miss; writes one
//                            source descriptor per row and the compacted list of missing rows
//   hit copy  (main stream)  rows from the local shard or the replica cache, 128-bit vectors,
//                            output walked flat so that stores are dense
//   miss copy (side stream)  rows read straight from pinned host memory over PCIe, started as
//                            soon as the classification is done and joined before the call ends
#include "spp_common.h"
#include "spp_device.h"
#include "spp_rowcopy.h"

#include <stdlib.h>

namespace spp {

struct ClassifyArgs {
    const int32_t* ids;
    int64_t        n;
    const int64_t* n_ptr;
    int64_t        N, lo, hi;
    const unsigned long long* tab;     // null: no cache
    uint32_t       mask;
    int            shift;
    int64_t        limit;              // slots in use
    int64_t*       desc;
    int32_t*       misslist;
    unsigned long long* counters;      // [0] local, [1] cache hit, [2] miss, [3] bad id
    unsigned long long* totals;        // context-wide running sums: [3] calls, [4] local, [5] cache hit, [6] miss
};

__global__ void gather_zero_kernel(unsigned long long* counters) {
    if (threadIdx.x < 8) counters[threadIdx.x] = 0ull;
}

constexpr int kClsPer = 8;             // ids per thread: a workgroup classifies 2048 consecutive ids per round

// One workgroup classifies a run of consecutive ids, then reserves room for all of its misses in
// the miss list with a single atomic (ranks inside the workgroup come from a scan), so the list
// counter sees one atomic per 2048 ids instead of one per wavefront.
__global__ void __launch_bounds__(kBlock) classify_kernel(ClassifyArgs a) {
    __shared__ int scan_lds[4];
    __shared__ unsigned long long base_lds;
    const int64_t n = a.n_ptr ? *a.n_ptr : a.n;
    constexpr int64_t kChunk = (int64_t)kBlock * kClsPer;
    int n_local = 0, n_hit = 0;
    for (int64_t base = (int64_t)blockIdx.x * kChunk; base < n; base += (int64_t)gridDim.x * kChunk) {
        uint32_t missbits = 0;
#pragma unroll
        for (int k = 0; k < kClsPer; ++k) {
            const int64_t i = base + (int64_t)k * kBlock + threadIdx.x;
            if (i >= n) continue;
            const int64_t g = a.ids[i];
            int64_t d = make_desc(kTagSkip, 0);
            if (g < 0 || g >= a.N) {
                atomicOr(&a.counters[3], 1ull);
            } else if (g >= a.lo && g < a.hi) {
                d = make_desc(kTagLocal, g - a.lo);
                ++n_local;
            } else {
                uint32_t slot = 0;
                const bool found = a.tab && table_find(a.tab, a.mask, a.shift, (uint32_t)g, slot) >= 0 &&
                                   (int64_t)slot < a.limit;
                if (found) { d = make_desc(kTagCache, slot); ++n_hit; }
                else       { d = make_desc(kTagMiss, g < a.lo ? g : g - (a.hi - a.lo)); missbits |= 1u << k; }
            }
            a.desc[i] = d;
        }
        int total;
        const int ex = block_exclusive_scan(__popc(missbits), scan_lds, total);
        if (total > 0) {
            if (threadIdx.x == 0) {
                base_lds = atomicAdd(&a.counters[2], (unsigned long long)total);
                atomicAdd(&a.totals[6], (unsigned long long)total);
            }
            __syncthreads();
            unsigned long long pos = base_lds + (unsigned long long)ex;
#pragma unroll
            for (int k = 0; k < kClsPer; ++k)
                if (missbits & (1u << k)) a.misslist[pos++] = (int32_t)(base + (int64_t)k * kBlock + threadIdx.x);
            __syncthreads();                      // base_lds is reused by the next round
        }
    }
    const int tl = block_reduce_sum(n_local, scan_lds);
    const int th = block_reduce_sum(n_hit, scan_lds);
    if (threadIdx.x == 0) {
        if (tl) { atomicAdd(&a.counters[0], (unsigned long long)tl); atomicAdd(&a.totals[4], (unsigned long long)tl); }
        if (th) { atomicAdd(&a.counters[1], (unsigned long long)th); atomicAdd(&a.totals[5], (unsigned long long)th); }
        if (blockIdx.x == 0) atomicAdd(&a.totals[3], 1ull);
    }
}

template <int V>
static void launch_hit(int grid, hipStream_t st, const int64_t* desc, int64_t n, const int64_t* n_ptr,
                       const void* local, const void* cache, int64_t row_bytes, void* out) {
    gather_hit_kernel<V><<<grid, kBlock, 0, st>>>(desc, n, n_ptr, (const char*)local, (const char*)cache,
                                                  (uint32_t)(row_bytes / V), (char*)out);
}

template <int V>
static void launch_indexed(int grid, hipStream_t st, const void* src, const int64_t* rowidx_or_desc,
                           const int32_t* list, int64_t count, const int64_t* count_ptr, int64_t row_bytes,
                           void* out) {
    rows_indexed_kernel<V><<<grid, kBlock, 0, st>>>((const char*)src, rowidx_or_desc, list, count, count_ptr,
                                                    (uint32_t)(row_bytes / V), (char*)out);
}

// Device-visible address of a row store that is either device memory or pinned host memory.
static int device_view(const void* p, const void** out) {
    *out = p;
    if (!p) return SPP_OK;
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        set_error("the remote row store is neither device memory nor pinned host memory (%s)", hipGetErrorString(e));
        return SPP_E_ARG;
    }
    if (attr.type == hipMemoryTypeHost) {
        void* dp = nullptr;
        e = hipHostGetDevicePointer(&dp, const_cast<void*>(p), 0);
        if (e != hipSuccess) { set_error("hipHostGetDevicePointer: %s", hipGetErrorString(e)); return SPP_E_HIP; }
        *out = dp;
    } else if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) {
        set_error("the remote row store is ordinary pageable host memory; pin it (hipHostMalloc)");
        return SPP_E_ARG;
    }
    return SPP_OK;
}

int copy_rows_indexed(hipStream_t st, const void* src, const int64_t* d_rowidx, int64_t n, int64_t row_bytes,
                      void* d_out, int num_cu) {
    if (n <= 0) return SPP_OK;
    const void* dsrc = nullptr;
    SPP_TRY(device_view(src, &dsrc));
    const int V = pick_vec(row_bytes, dsrc, d_out, nullptr, nullptr);
    const int64_t vecs = n * (row_bytes / V);
    int64_t need = (vecs + kBlock * kCopyUnroll - 1) / (kBlock * kCopyUnroll);
    const int grid = (int)(need < (int64_t)num_cu * 8 ? need : (int64_t)num_cu * 8);
    switch (V) {
        case 16: launch_indexed<16>(grid, st, dsrc, d_rowidx, nullptr, n, nullptr, row_bytes, d_out); break;
        case 8:  launch_indexed<8>(grid, st, dsrc, d_rowidx, nullptr, n, nullptr, row_bytes, d_out); break;
        case 4:  launch_indexed<4>(grid, st, dsrc, d_rowidx, nullptr, n, nullptr, row_bytes, d_out); break;
        default: launch_indexed<2>(grid, st, dsrc, d_rowidx, nullptr, n, nullptr, row_bytes, d_out); break;
    }
    SPP_HIP(hipGetLastError());
    return SPP_OK;
}

}  // namespace spp

extern "C" int spp_gather_features(spp_ctx* ctx, const spp_cache* cache, const void* d_local,
                                   int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D,
                                   int32_t elem_bytes, const int32_t* d_node_ids, int64_t n,
                                   const int64_t* d_n, void* d_out, spp_gather_stats* stats, uint32_t flags) {
    using namespace spp;
    SPP_CHECK(ctx, SPP_E_ARG, "spp_gather_features: ctx is null");
    SPP_CHECK(n >= 0 && N > 0 && lo >= 0 && lo <= hi && hi <= N, SPP_E_ARG,
              "spp_gather_features: n = %lld, range [%lld, %lld) of N = %lld", (long long)n, (long long)lo, (long long)hi, (long long)N);
    SPP_CHECK(D >= 1 && elem_bytes >= 1, SPP_E_ARG, "spp_gather_features: D = %d, elem_bytes = %d", D, elem_bytes);
    const int64_t row_bytes = (int64_t)D * elem_bytes;
    SPP_CHECK(row_bytes % 2 == 0, SPP_E_ARG, "spp_gather_features: row size %lld is odd", (long long)row_bytes);
    SPP_CHECK(n == 0 || (d_node_ids && d_out), SPP_E_ARG, "spp_gather_features: null ids or output");
    SPP_CHECK(hi == lo || d_local || n == 0, SPP_E_ARG, "spp_gather_features: local shard is null");
    if (cache) {
        SPP_CHECK(cache->lo == lo && cache->hi == hi && cache->N == N, SPP_E_ARG,
                  "spp_gather_features: the cache was built for another partition range");
        SPP_CHECK(cache->rows != nullptr || cache->limit == 0, SPP_E_ARG, "spp_gather_features: the cache holds no rows");
        SPP_CHECK(cache->row_bytes == row_bytes || cache->limit == 0, SPP_E_ARG,
                  "spp_gather_features: cache rows are %lld bytes, requested %lld", (long long)cache->row_bytes, (long long)row_bytes);
    }
    SPP_HIP(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;
    const void* dremote = nullptr;
    SPP_TRY(device_view(remote, &dremote));
    SPP_TRY(ctx->gcount.reserve(8 * sizeof(unsigned long long)));
    unsigned long long* counters = ctx->gcount.as<unsigned long long>();
    if (n > 0) {
        SPP_TRY(ctx->srcdesc.reserve((size_t)n * sizeof(int64_t)));
        SPP_TRY(ctx->misslist.reserve((size_t)n * sizeof(int32_t)));
    }
    gather_zero_kernel<<<1, 64, 0, st>>>(counters);
    if (n > 0) {
        ClassifyArgs a;
        a.ids = d_node_ids; a.n = n; a.n_ptr = d_n; a.N = N; a.lo = lo; a.hi = hi;
        a.tab = cache && cache->limit > 0 ? reinterpret_cast<const unsigned long long*>(cache->table) : nullptr;
        a.mask = cache ? cache->table_mask : 0; a.shift = cache ? cache->table_shift : 0;
        a.limit = cache ? cache->limit : 0;
        a.desc = ctx->srcdesc.as<int64_t>(); a.misslist = ctx->misslist.as<int32_t>(); a.counters = counters;
        a.totals = reinterpret_cast<unsigned long long*>(ctx->totals);
        const int64_t cneed = (n + kBlock * kClsPer - 1) / (kBlock * kClsPer);
        const int cgrid = (int)(cneed < (int64_t)ctx->num_cu * 8 ? cneed : (int64_t)ctx->num_cu * 8);
        {
            ScopedTimer tc(ctx, SPP_T_GATHER_CLASSIFY, st);
            classify_kernel<<<cgrid, kBlock, 0, st>>>(a);
        }
        const void* crow = cache ? cache->rows : nullptr;
        const int V = pick_vec(row_bytes, d_local, crow, dremote, d_out);
        const int64_t vecs = n * (row_bytes / V);
        const int64_t need = (vecs + kBlock * kCopyUnroll - 1) / (kBlock * kCopyUnroll);
        const int grid = (int)(need < (int64_t)ctx->num_cu * 16 ? need : (int64_t)ctx->num_cu * 16);
        // The miss kernel is kept to a few workgroups on purpose: 64 of them already saturate
        // the PCIe link, and every CU that hosts host-memory loads serves other kernels slowly.
        int64_t mcap = 64;
        if (const char* env = getenv("SPP_MISS_BLOCKS")) { const long v = atol(env); if (v > 0) mcap = v; }
        const int mgrid = (int)(need < mcap ? need : mcap);
        // miss path on the side stream, after the classification
        if (dremote) {
            SPP_HIP(hipEventRecord(ctx->ev_fork, st));
            SPP_HIP(hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0));
            {
                ScopedTimer tm(ctx, SPP_T_GATHER_MISS, ctx->side);
                const int64_t* miss_count = reinterpret_cast<const int64_t*>(counters + 2);
                switch (V) {
                    case 16: launch_indexed<16>(mgrid, ctx->side, dremote, a.desc, a.misslist, 0, miss_count, row_bytes, d_out); break;
                    case 8:  launch_indexed<8>(mgrid, ctx->side, dremote, a.desc, a.misslist, 0, miss_count, row_bytes, d_out); break;
                    case 4:  launch_indexed<4>(mgrid, ctx->side, dremote, a.desc, a.misslist, 0, miss_count, row_bytes, d_out); break;
                    default: launch_indexed<2>(mgrid, ctx->side, dremote, a.desc, a.misslist, 0, miss_count, row_bytes, d_out); break;
                }
            }
            SPP_HIP(hipEventRecord(ctx->ev_join, ctx->side));
        }
        {
            ScopedTimer th(ctx, SPP_T_GATHER_HIT, st);
            switch (V) {
                case 16: launch_hit<16>(grid, st, a.desc, n, d_n, d_local, crow, row_bytes, d_out); break;
                case 8:  launch_hit<8>(grid, st, a.desc, n, d_n, d_local, crow, row_bytes, d_out); break;
                case 4:  launch_hit<4>(grid, st, a.desc, n, d_n, d_local, crow, row_bytes, d_out); break;
                default: launch_hit<2>(grid, st, a.desc, n, d_n, d_local, crow, row_bytes, d_out); break;
            }
        }
        if (dremote) SPP_HIP(hipStreamWaitEvent(st, ctx->ev_join, 0));
    }
    SPP_HIP(hipGetLastError());
    int64_t* hp = ctx->h_pinned + 40;
    SPP_HIP(hipMemcpyAsync(hp, counters, 4 * sizeof(int64_t), hipMemcpyDeviceToHost, st));
    ctx->h_pinned[48] = row_bytes;
    ctx->h_pinned[49] = dremote ? 1 : 0;
    if (flags & SPP_SYNC) {
        SPP_HIP(hipStreamSynchronize(st));
        return spp_gather_last_stats(ctx, stats);
    }
    return SPP_OK;
}

extern "C" int spp_gather_last_stats(spp_ctx* ctx, spp_gather_stats* stats) {
    SPP_CHECK(ctx, SPP_E_ARG, "spp_gather_last_stats: ctx is null");
    const int64_t* hp = ctx->h_pinned + 40;
    if (stats) {
        stats->n_local = hp[0]; stats->n_cache_hit = hp[1]; stats->n_miss = hp[2];
        stats->miss_bytes = hp[2] * ctx->h_pinned[48];
    }
    SPP_CHECK(hp[3] == 0, SPP_E_ARG, "spp_gather_features: a vertex id lies outside [0, N); its row was left untouched");
    SPP_CHECK(hp[2] == 0 || ctx->h_pinned[49] != 0, SPP_E_ARG,
              "spp_gather_features: %lld rows missed but no remote store was given; they were left untouched", (long long)hp[2]);
    return SPP_OK;
}
