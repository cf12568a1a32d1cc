// VIP-ranked replica cache (Secs. 3.2, 4.2): rank the remote vertices by decreasing score, keep
// the first floor(alpha*N/K), build the id -> slot table, copy their rows from the remote store.
//
// Candidates (remote, score > 0) are compacted in ascending id order by a grid scan, packed as
// (~score bits) << 32 | id, and stably radix-sorted on the score bits only: positive floats order
// like their bit patterns, the complement turns that into descending score, and stability keeps
// ascending id among equal scores.
#include "spp_common.h"
#include "spp_device.h"
#include "spp_rowcopy.h"

#include <math.h>
#include <new>

namespace spp {

struct CandIn {
    const float* score; int64_t lo, hi;
    __device__ int operator()(int64_t u) const { return ((u < lo || u >= hi) && score[u] > 0.0f) ? 1 : 0; }
};
struct CandOut {
    const float* score; uint64_t* keys;
    __device__ void operator()(int64_t u, int ex, int v) const {
        if (v) keys[(uint32_t)ex] = ((uint64_t)(~__float_as_uint(score[u])) << 32) | (uint32_t)u;
    }
};
struct CandFin {
    int64_t* total;
    __device__ void operator()(int t) const { *total = (int64_t)(uint32_t)t; }
};

__global__ void __launch_bounds__(kBlock) cache_fill_kernel(const uint64_t* __restrict__ sorted, int64_t n,
                                                            int64_t lo, int64_t hi, int32_t* __restrict__ ids,
                                                            int64_t* __restrict__ rowidx,
                                                            unsigned long long* __restrict__ tab, uint32_t mask,
                                                            int shift) {
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r >= n) return;
    const uint32_t id = (uint32_t)sorted[r];
    ids[r] = (int32_t)id;
    rowidx[r] = (int64_t)id < lo ? (int64_t)id : (int64_t)id - (hi - lo);
    table_insert_min(tab, mask, shift, id, (uint32_t)r);
}

__global__ void fill_table_kernel(unsigned long long* p, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = ~0ull;
}

__global__ void __launch_bounds__(kBlock) cache_lookup_kernel(const unsigned long long* __restrict__ tab,
                                                              uint32_t mask, int shift, int64_t limit,
                                                              const int32_t* __restrict__ ids, int64_t n,
                                                              int32_t* __restrict__ out) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        uint32_t slot = 0;
        const int32_t g = ids[i];
        const bool found = tab && g >= 0 && table_find(tab, mask, shift, (uint32_t)g, slot) >= 0 && (int64_t)slot < limit;
        out[i] = found ? (int32_t)slot : -1;
    }
}

// Empirical access frequencies (Sec. 3.2, "sim." and "oracle" policies): one count per listed id.
// Ids of one minibatch are distinct and the lists of a call are few, so the float atomics rarely
// meet on one address.
struct CountLists {
    const int32_t* ids[SPP_MAX_GATHER_LISTS];
    int64_t        n[SPP_MAX_GATHER_LISTS];
    const int64_t* n_ptr[SPP_MAX_GATHER_LISTS];
};
__global__ void clear_flag_kernel(int* flag) { if (threadIdx.x == 0) *flag = 0; }

__global__ void __launch_bounds__(kBlock) access_count_kernel(CountLists l, int64_t N, float* __restrict__ count,
                                                              int* __restrict__ bad) {
    const int j = blockIdx.y;
    int64_t n = l.n_ptr[j] ? *l.n_ptr[j] : l.n[j];
    if (n > l.n[j]) n = l.n[j];                       // never beyond what the caller's buffer holds
    const int32_t* __restrict__ ids = l.ids[j];
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        const int64_t g = ids[i];
        if (g < 0 || g >= N) atomicOr(bad, 1);
        else unsafeAtomicAdd(&count[g], 1.0f);
    }
}

}  // namespace spp

extern "C" int spp_access_count(spp_ctx* ctx, const spp_id_list* lists, int32_t n_lists, int64_t N, float* d_count,
                                uint32_t flags) {
    using namespace spp;
    SPP_CHECK(ctx && d_count && (lists || n_lists == 0), SPP_E_ARG, "spp_access_count: null argument");
    SPP_CHECK(n_lists >= 0 && n_lists <= SPP_MAX_GATHER_LISTS, SPP_E_ARG, "spp_access_count: %d lists (at most %d)",
              n_lists, SPP_MAX_GATHER_LISTS);
    SPP_CHECK(N > 0, SPP_E_ARG, "spp_access_count: N = %lld", (long long)N);
    if (n_lists == 0) return SPP_OK;
    CountLists l;
    memset(&l, 0, sizeof(l));
    int64_t nmax = 0;
    for (int j = 0; j < n_lists; ++j) {
        SPP_CHECK(lists[j].n >= 0 && (lists[j].d_ids || lists[j].n == 0), SPP_E_ARG, "spp_access_count: list %d", j);
        l.ids[j] = lists[j].d_ids; l.n[j] = lists[j].n; l.n_ptr[j] = lists[j].d_n;
        if (lists[j].n > nmax) nmax = lists[j].n;
    }
    if (nmax == 0) return SPP_OK;
    SPP_HIP(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;
    SPP_TRY(ctx->partials.reserve(256));
    int* d_bad = ctx->partials.as<int>();
    clear_flag_kernel<<<1, 64, 0, st>>>(d_bad);
    const int64_t need = (nmax + kBlock - 1) / kBlock;
    const int64_t lim = (int64_t)ctx->num_cu * 8 / n_lists + 1;
    access_count_kernel<<<dim3((unsigned)(need < lim ? need : lim), n_lists), kBlock, 0, st>>>(l, N, d_count, d_bad);
    SPP_HIP(hipGetLastError());
    if (flags & SPP_SYNC) {
        int* hb = reinterpret_cast<int*>(ctx->h_pinned + 60);
        SPP_HIP(hipMemcpyAsync(hb, d_bad, sizeof(int), hipMemcpyDeviceToHost, st));
        SPP_HIP(hipStreamSynchronize(st));
        SPP_CHECK(*hb == 0, SPP_E_ARG, "spp_access_count: an id lies outside [0, N); it was skipped");
    }
    return SPP_OK;
}

extern "C" int spp_build_vip_cache(spp_ctx* ctx, const float* d_score, int64_t N, int64_t lo, int64_t hi,
                                   int32_t K, double alpha, const void* remote, int32_t D,
                                   int32_t elem_bytes, int32_t* d_cache_ids, int64_t* n_cached,
                                   spp_cache** out) {
    using namespace spp;
    SPP_CHECK(ctx && d_score && n_cached && out, SPP_E_ARG, "spp_build_vip_cache: null argument");
    *out = nullptr; *n_cached = 0;
    SPP_CHECK(N > 0 && N <= 0x7FFFFFFFll && lo >= 0 && lo <= hi && hi <= N, SPP_E_ARG,
              "spp_build_vip_cache: range [%lld, %lld) of N = %lld", (long long)lo, (long long)hi, (long long)N);
    SPP_CHECK(K >= 1 && alpha >= 0.0 && alpha == alpha, SPP_E_ARG, "spp_build_vip_cache: K = %d, alpha = %g", K, alpha);
    SPP_CHECK(D >= 1 && elem_bytes >= 1 && ((int64_t)D * elem_bytes) % 2 == 0, SPP_E_ARG,
              "spp_build_vip_cache: D = %d, elem_bytes = %d", D, elem_bytes);
    const int64_t C = (int64_t)floor(alpha * (double)N / (double)K);
    SPP_CHECK(C == 0 || d_cache_ids, SPP_E_ARG, "spp_build_vip_cache: d_cache_ids is null");
    SPP_HIP(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;

    spp_cache* c = new (std::nothrow) spp_cache();
    SPP_CHECK(c != nullptr, SPP_E_OOM, "spp_build_vip_cache: out of host memory");
    c->device = ctx->device; c->N = N; c->lo = lo; c->hi = hi; c->row_bytes = (int64_t)D * elem_bytes;

    int rc = SPP_OK;
    uint64_t *ka = nullptr, *kb = nullptr, *sorted = nullptr;
    int64_t* d_tmp = nullptr;          // [0] = N (scan length), [1] = number of candidates
    int* partial = nullptr;
    int64_t* rowidx = nullptr;
    const int scan_grid = 1024;
    const int64_t max_cand = N - (hi - lo);
    int64_t ncand = 0, keep = 0;

    auto fail = [&](int code) { rc = code; };
    do {
        if (C == 0 || max_cand == 0) break;
        if (hipMalloc(&ka, (size_t)max_cand * sizeof(uint64_t)) != hipSuccess ||
            hipMalloc(&kb, (size_t)max_cand * sizeof(uint64_t)) != hipSuccess ||
            hipMalloc(&d_tmp, 2 * sizeof(int64_t)) != hipSuccess ||
            hipMalloc(&partial, scan_grid * sizeof(int)) != hipSuccess) {
            set_error("spp_build_vip_cache: out of device memory for %lld candidates", (long long)max_cand);
            fail(SPP_E_OOM); break;
        }
        int64_t init[2] = {N, 0};
        if (hipMemcpy(d_tmp, init, sizeof(init), hipMemcpyHostToDevice) != hipSuccess) { set_error("spp_build_vip_cache: copy failed"); fail(SPP_E_HIP); break; }
        grid_scan(st, scan_grid, d_tmp, CandIn{d_score, lo, hi}, CandOut{d_score, ka}, CandFin{d_tmp + 1}, partial);
        if (hipMemcpyAsync(&ncand, d_tmp + 1, sizeof(int64_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess) { set_error("spp_build_vip_cache: candidate scan failed: %s", hipGetErrorString(hipGetLastError())); fail(SPP_E_HIP); break; }
        if (ncand == 0) break;
        rc = radix_sort_u64(ctx, ka, kb, ncand, 32, 64, &sorted);
        if (rc != SPP_OK) break;
        keep = ncand < C ? ncand : C;
        const uint32_t cap = next_pow2((uint64_t)(2 * keep > 1024 ? 2 * keep : 1024));
        int shift = 32;
        for (uint32_t t = cap; t > 1; t >>= 1) --shift;
        c->table_mask = cap - 1; c->table_shift = shift;
        if (hipMalloc(&c->table, (size_t)cap * sizeof(uint64_t)) != hipSuccess ||
            hipMalloc(&rowidx, (size_t)keep * sizeof(int64_t)) != hipSuccess) {
            set_error("spp_build_vip_cache: out of device memory for the id table"); fail(SPP_E_OOM); break;
        }
        fill_table_kernel<<<ctx->num_cu * 4, kBlock, 0, st>>>(reinterpret_cast<unsigned long long*>(c->table), cap);
        cache_fill_kernel<<<(unsigned)((keep + kBlock - 1) / kBlock), kBlock, 0, st>>>(
            sorted, keep, lo, hi, d_cache_ids, rowidx, reinterpret_cast<unsigned long long*>(c->table), c->table_mask, shift);
        if (remote) {
            if (hipMalloc(&c->rows, (size_t)keep * (size_t)c->row_bytes) != hipSuccess) {
                set_error("spp_build_vip_cache: out of device memory for %lld cached rows", (long long)keep); fail(SPP_E_OOM); break;
            }
            rc = copy_rows_indexed(st, remote, rowidx, keep, c->row_bytes, c->rows, ctx->num_cu);
            if (rc != SPP_OK) break;
        }
        if (hipStreamSynchronize(st) != hipSuccess) { set_error("spp_build_vip_cache: %s", hipGetErrorString(hipGetLastError())); fail(SPP_E_HIP); break; }
    } while (0);

    if (ka) (void)hipFree(ka);
    if (kb) (void)hipFree(kb);
    if (d_tmp) (void)hipFree(d_tmp);
    if (partial) (void)hipFree(partial);
    if (rowidx) (void)hipFree(rowidx);
    if (rc != SPP_OK) { spp_cache_destroy(c); return rc; }
    c->n_rows = keep; c->limit = keep;
    *n_cached = keep;
    *out = c;
    return SPP_OK;
}

extern "C" void spp_cache_destroy(spp_cache* c) {
    if (!c) return;
    if (hipSetDevice(c->device) != hipSuccess) { (void)hipGetLastError(); delete c; return; }   // runtime already shut down
    (void)hipDeviceSynchronize();      // a gather that still reads the cache may be in flight
    if (c->table) (void)hipFree(c->table);
    if (c->rows) (void)hipFree(c->rows);
    delete c;
}

extern "C" int spp_cache_set_limit(spp_cache* c, int64_t n_slots) {
    SPP_CHECK(c, SPP_E_ARG, "spp_cache_set_limit: cache is null");
    SPP_CHECK(n_slots <= c->n_rows, SPP_E_ARG, "spp_cache_set_limit: %lld slots asked, %lld built", (long long)n_slots, (long long)c->n_rows);
    c->limit = n_slots < 0 ? c->n_rows : n_slots;
    return SPP_OK;
}

extern "C" int spp_cache_lookup(spp_ctx* ctx, const spp_cache* c, const int32_t* d_ids, int64_t n,
                                int32_t* d_slot_out) {
    using namespace spp;
    SPP_CHECK(ctx && c && (n == 0 || (d_ids && d_slot_out)), SPP_E_ARG, "spp_cache_lookup: null argument");
    if (n == 0) return SPP_OK;
    SPP_HIP(hipSetDevice(ctx->device));
    const int64_t need = (n + kBlock - 1) / kBlock;
    const int grid = (int)(need < (int64_t)ctx->num_cu * 8 ? need : (int64_t)ctx->num_cu * 8);
    // an empty cache has no table: every id misses
    cache_lookup_kernel<<<grid, kBlock, 0, ctx->stream>>>(reinterpret_cast<const unsigned long long*>(c->table),
                                                          c->table_mask, c->table_shift, c->limit, d_ids, n, d_slot_out);
    SPP_HIP(hipGetLastError());
    return SPP_OK;
}
