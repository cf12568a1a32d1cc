// Graph handle: wraps the caller's CSR and, on request, builds the in-lists (the transposed CSR)
// that the pull form of Proposition 1, eq. (2), walks: for every u the ascending list of v with
// u in adj(v).  Built once per graph by a stable radix sort of the packed edge keys.
#include "spp_common.h"
#include "spp_device.h"

#include <algorithm>
#include <new>
#include <vector>

namespace spp {

// key[e] = (u << 32) | v for the e-th edge v -> u of the CSR; one wavefront walks one row at a time.
__global__ void __launch_bounds__(kBlock) edge_keys_kernel(int64_t N, int64_t M, const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col,
                                                           uint64_t* __restrict__ keys, int* __restrict__ bad) {
    const int lane = lane_id();
    const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    for (int64_t v = wave; v < N; v += nwaves) {
        const int64_t b = rowptr[v], e = rowptr[v + 1];
        if (b < 0 || e > M || b > e) { *bad = 1; continue; }
        for (int64_t i = b + lane; i < e; i += kWave) {
            const int32_t u = col[i];
            if (u < 0 || u >= N) *bad = 1;          // reported to the caller; the key stays in range
            keys[i] = ((uint64_t)(uint32_t)(u < 0 || u >= N ? 0 : u) << 32) | (uint32_t)v;
        }
    }
}

// Every kernel of the library indexes with these arrays, so they are checked once here: offsets
// monotone inside [0, M], column ids inside [0, N).
__global__ void __launch_bounds__(kBlock) validate_csr_kernel(int64_t N, int64_t M, const int64_t* __restrict__ rowptr,
                                                              const int32_t* __restrict__ col, int* __restrict__ bad) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    for (int64_t v = t; v < N; v += stride) {
        const int64_t b = rowptr[v], e = rowptr[v + 1];
        if (b < 0 || e > M || b > e) *bad = 1;
    }
    for (int64_t i = t; i < M; i += stride) {
        const int32_t u = col[i];
        if (u < 0 || u >= N) *bad = 1;
    }
}

// From the sorted keys: in_col[e] = v, and in_rowptr[r] = first e whose u is >= r (rows after the
// last u keep the value M they were filled with).
__global__ void __launch_bounds__(kBlock) in_lists_kernel(const uint64_t* __restrict__ keys, int64_t M,
                                                          int64_t N, int32_t* __restrict__ in_col,
                                                          int64_t* __restrict__ in_rowptr) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < M; e += stride) {
        const uint64_t k = keys[e];
        in_col[e] = (int32_t)(uint32_t)k;
        const int64_t u = (int64_t)(k >> 32);
        const int64_t uprev = e > 0 ? (int64_t)(keys[e - 1] >> 32) : -1;
        for (int64_t r = uprev + 1; r <= u; ++r) in_rowptr[r] = e;
    }
}

__global__ void fill_i64_kernel(int64_t* p, int64_t n, int64_t v) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

// blk_row[b] = first in-row whose list starts at or after edge b * kVipChunk (b < nblk); blk_row[nblk] = N.
__global__ void __launch_bounds__(kBlock) block_rows_kernel(const int64_t* __restrict__ in_rowptr, int64_t N,
                                                            int64_t nblk, int32_t* __restrict__ blk_row) {
    const int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (b > nblk) return;
    if (b == nblk) { blk_row[b] = (int32_t)N; return; }
    const int64_t want = b * kVipChunk;
    int64_t lo = 0, hi = N;                       // first r in [0, N] with in_rowptr[r] >= want
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (in_rowptr[mid] >= want) hi = mid; else lo = mid + 1;
    }
    blk_row[b] = (int32_t)lo;
}

// Appends every in-row longer than kVipChunk (a hub) to the list, with its length.
__global__ void __launch_bounds__(kBlock) find_hubs_kernel(const int64_t* __restrict__ in_rowptr, int64_t N,
                                                           int32_t* hub_rows, int64_t* hub_len,
                                                           unsigned long long* count, int64_t cap) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x; r < N; r += stride) {
        const int64_t len = in_rowptr[r + 1] - in_rowptr[r];
        if (len > kVipChunk) {
            const unsigned long long k = atomicAdd(count, 1ull);
            if ((int64_t)k < cap) { hub_rows[k] = (int32_t)r; hub_len[k] = len; }
        }
    }
}

static int build_in_lists(spp_ctx* ctx, spp_graph* g) {
    hipStream_t st = ctx->stream;
    const int64_t N = g->N, M = g->M;
    const int grid = ctx->num_cu * 8;
    SPP_HIP(hipMalloc(&g->in_rowptr, (size_t)(N + 1) * sizeof(int64_t)));
    SPP_HIP(hipMalloc(&g->in_col, (size_t)(M > 0 ? M : 1) * sizeof(int32_t)));
    fill_i64_kernel<<<grid, kBlock, 0, st>>>(g->in_rowptr, N + 1, M);
    if (M > 0) {
        uint64_t *ka = nullptr, *kb = nullptr, *sorted = nullptr;
        SPP_HIP(hipMalloc(&ka, (size_t)M * sizeof(uint64_t)));
        hipError_t e = hipMalloc(&kb, (size_t)M * sizeof(uint64_t));
        if (e != hipSuccess) { (void)hipFree(ka); set_error("in-lists: out of device memory for sort keys"); return SPP_E_OOM; }
        int* d_bad = nullptr;
        e = hipMalloc(&d_bad, sizeof(int));
        if (e != hipSuccess) { (void)hipFree(ka); (void)hipFree(kb); set_error("in-lists: out of device memory"); return SPP_E_OOM; }
        (void)hipMemsetAsync(d_bad, 0, sizeof(int), st);
        edge_keys_kernel<<<grid, kBlock, 0, st>>>(N, M, g->rowptr, g->col, ka, d_bad);
        int bits = 1;
        while (((int64_t)1 << bits) < N) ++bits;
        int rc = radix_sort_u64(ctx, ka, kb, M, 32, 32 + bits, &sorted);
        int bad = 0;
        if (rc == SPP_OK && hipMemcpy(&bad, d_bad, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) bad = 1;
        (void)hipFree(d_bad);
        if (rc == SPP_OK && bad) { set_error("spp_graph_create: rowptr is not monotone within [0, M] or a column index lies outside [0, N)"); rc = SPP_E_ARG; }
        if (rc == SPP_OK) {
            in_lists_kernel<<<grid, kBlock, 0, st>>>(sorted, M, N, g->in_col, g->in_rowptr);
            hipError_t e2 = hipStreamSynchronize(st);
            if (e2 != hipSuccess) { set_error("in-lists: %s", hipGetErrorString(e2)); rc = SPP_E_HIP; }
        }
        (void)hipFree(ka); (void)hipFree(kb);
        SPP_TRY(rc);
    }
    // workgroup -> row ranges of the pull kernel
    g->nblk = M > 0 ? (M + kVipChunk - 1) / kVipChunk : 1;
    SPP_HIP(hipMalloc(&g->blk_row, (size_t)(g->nblk + 1) * sizeof(int32_t)));
    block_rows_kernel<<<(unsigned)((g->nblk + 1 + kBlock - 1) / kBlock), kBlock, 0, st>>>(g->in_rowptr, N, g->nblk, g->blk_row);
    // hubs
    const int64_t cap = M / kVipChunk + 1;
    int32_t* d_rows = nullptr; int64_t* d_len = nullptr; unsigned long long* d_cnt = nullptr;
    SPP_HIP(hipMalloc(&d_rows, (size_t)cap * sizeof(int32_t)));
    SPP_HIP(hipMalloc(&d_len, (size_t)cap * sizeof(int64_t)));
    SPP_HIP(hipMalloc(&d_cnt, sizeof(unsigned long long)));
    fill_i64_kernel<<<1, 64, 0, st>>>(reinterpret_cast<int64_t*>(d_cnt), 1, 0);
    find_hubs_kernel<<<grid, kBlock, 0, st>>>(g->in_rowptr, N, d_rows, d_len, d_cnt, cap);
    unsigned long long nh = 0;
    SPP_HIP(hipMemcpyAsync(&nh, d_cnt, sizeof(nh), hipMemcpyDeviceToHost, st));
    SPP_HIP(hipStreamSynchronize(st));
    g->nhub = (int64_t)nh;
    g->nslices = 0;
    if (nh > 0) {
        std::vector<int32_t> rows(nh);
        std::vector<int64_t> len(nh);
        SPP_HIP(hipMemcpy(rows.data(), d_rows, nh * sizeof(int32_t), hipMemcpyDeviceToHost));
        SPP_HIP(hipMemcpy(len.data(), d_len, nh * sizeof(int64_t), hipMemcpyDeviceToHost));
        std::vector<size_t> order(nh);
        for (size_t i = 0; i < nh; ++i) order[i] = i;
        std::sort(order.begin(), order.end(), [&](size_t a, size_t b) { return rows[a] < rows[b]; });
        std::vector<int32_t> srows(nh);
        std::vector<int64_t> sptr(nh + 1, 0);
        for (size_t i = 0; i < nh; ++i) {
            srows[i] = rows[order[i]];
            sptr[i + 1] = sptr[i] + (len[order[i]] + kHubSlice - 1) / kHubSlice;
        }
        g->nslices = sptr[nh];
        SPP_HIP(hipMalloc(&g->hub_rows, nh * sizeof(int32_t)));
        SPP_HIP(hipMalloc(&g->hub_slice_ptr, (nh + 1) * sizeof(int64_t)));
        SPP_HIP(hipMemcpy(g->hub_rows, srows.data(), nh * sizeof(int32_t), hipMemcpyHostToDevice));
        SPP_HIP(hipMemcpy(g->hub_slice_ptr, sptr.data(), (nh + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    }
    (void)hipFree(d_rows); (void)hipFree(d_len); (void)hipFree(d_cnt);
    g->has_in = true;
    return SPP_OK;
}

}  // namespace spp

extern "C" int spp_graph_create(spp_ctx* ctx, int64_t N, int64_t M, const int64_t* d_rowptr,
                                const int32_t* d_col, uint32_t flags, spp_graph** out) {
    SPP_CHECK(ctx && out, SPP_E_ARG, "spp_graph_create: null argument");
    *out = nullptr;
    SPP_CHECK(N > 0 && N <= 0x7FFFFFFFll, SPP_E_ARG, "spp_graph_create: N = %lld out of range (int32 ids)", (long long)N);
    SPP_CHECK(M >= 0 && M < 0xFFFFFFFFll, SPP_E_ARG, "spp_graph_create: M = %lld out of range", (long long)M);
    SPP_CHECK(d_rowptr && (d_col || M == 0), SPP_E_ARG, "spp_graph_create: null CSR array");
    SPP_HIP(hipSetDevice(ctx->device));
    // the CSR must really describe M edges
    int64_t ends[2] = {-1, -1};
    SPP_HIP(hipMemcpy(&ends[0], d_rowptr, sizeof(int64_t), hipMemcpyDeviceToHost));
    SPP_HIP(hipMemcpy(&ends[1], d_rowptr + N, sizeof(int64_t), hipMemcpyDeviceToHost));
    SPP_CHECK(ends[0] == 0 && ends[1] == M, SPP_E_ARG, "spp_graph_create: rowptr[0] = %lld, rowptr[N] = %lld, M = %lld",
              (long long)ends[0], (long long)ends[1], (long long)M);
    spp_graph* g = new (std::nothrow) spp_graph();
    SPP_CHECK(g != nullptr, SPP_E_OOM, "spp_graph_create: out of host memory");
    g->device = ctx->device; g->N = N; g->M = M; g->rowptr = d_rowptr; g->col = d_col;
    {
        int* d_bad = nullptr;
        int bad = 0;
        hipError_t e = hipMalloc(&d_bad, sizeof(int));
        if (e == hipSuccess) e = hipMemsetAsync(d_bad, 0, sizeof(int), ctx->stream);
        if (e == hipSuccess) {
            spp::validate_csr_kernel<<<ctx->num_cu * 8, spp::kBlock, 0, ctx->stream>>>(N, M, d_rowptr, d_col, d_bad);
            e = hipMemcpyAsync(&bad, d_bad, sizeof(int), hipMemcpyDeviceToHost, ctx->stream);
        }
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (d_bad) (void)hipFree(d_bad);
        if (e != hipSuccess || bad) {
            if (e != hipSuccess) spp::set_error("spp_graph_create: %s", hipGetErrorString(e));
            else spp::set_error("spp_graph_create: rowptr is not monotone within [0, M] or a column id lies outside [0, N)");
            delete g;
            return e != hipSuccess ? SPP_E_HIP : SPP_E_ARG;
        }
    }
    if (flags & SPP_GRAPH_IN_LISTS) {
        int rc = spp::build_in_lists(ctx, g);
        if (rc != SPP_OK) { spp_graph_destroy(g); return rc; }
    }
    *out = g;
    return SPP_OK;
}

extern "C" void spp_graph_destroy(spp_graph* g) {
    if (!g) return;
    (void)hipSetDevice(g->device);
    (void)hipDeviceSynchronize();      // work that still reads the in-lists may be in flight
    if (g->in_rowptr) (void)hipFree(g->in_rowptr);
    if (g->in_col) (void)hipFree(g->in_col);
    if (g->blk_row) (void)hipFree(g->blk_row);
    if (g->hub_rows) (void)hipFree(g->hub_rows);
    if (g->hub_slice_ptr) (void)hipFree(g->hub_slice_ptr);
    delete g;
}
