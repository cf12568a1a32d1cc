// Graph handle: wraps the caller's CSR and, on request, builds the transposed structure that the
// pull form of Proposition 1, eq. (2), walks: the edges v -> u grouped by blocks of 2^14
// destination rows u and, inside a block, sorted by source v, 4 bytes per edge (the low 18 bits of
// the source and the row inside the block; a table says where each run of 2^18 sources starts in
// each block).  Built once per graph by a radix sort of the packed edge keys, then read back and
// compared with the keys before anything gathers through it.
#include "spp_common.h"
#include "spp_device.h"

#include <new>

namespace spp {

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

__global__ void fill_i64_kernel(int64_t* p, int64_t n, int64_t v) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

// key[e] = (row block of u, v, u inside its block) for the e-th edge v -> u of the CSR.
__global__ void __launch_bounds__(kBlock) tile_keys_kernel(int64_t N, const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col, int rbits, int vbits,
                                                           uint64_t* __restrict__ keys) {
    const int lane = lane_id();
    const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    const uint64_t rmask = (1ull << rbits) - 1;
    for (int64_t v = wave; v < N; v += nwaves) {
        const int64_t b = rowptr[v], e = rowptr[v + 1];
        for (int64_t i = b + lane; i < e; i += kWave) {
            const uint64_t u = (uint64_t)(uint32_t)col[i];          // validated at graph creation
            keys[i] = ((u >> rbits) << (vbits + rbits)) | ((uint64_t)v << rbits) | (u & rmask);
        }
    }
}

// From the sorted keys: the edge words, and first[g] = first e whose (row block, source chunk)
// index g = block * nch + chunk is >= g (indices after the last one keep the value M they were
// filled with).
__global__ void __launch_bounds__(kBlock) tile_lists_kernel(const uint64_t* __restrict__ keys, int64_t M, int rbits,
                                                            int vbits, int nch, uint32_t* __restrict__ t_edge,
                                                            int64_t* __restrict__ first) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const uint64_t rmask = (1ull << rbits) - 1, vmask = (1ull << vbits) - 1;
    auto index_of = [&](uint64_t k) {
        return (int64_t)(k >> (vbits + rbits)) * nch + (int64_t)(((k >> rbits) & vmask) >> kTileSrcLoBits);
    };
    for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < M; e += stride) {
        const uint64_t k = keys[e];
        const uint32_t v = (uint32_t)((k >> rbits) & vmask);
        t_edge[e] = ((v & ((1u << kTileSrcLoBits) - 1u)) << kTileRowBits) | (uint32_t)(k & rmask);
        const int64_t g = index_of(k);
        const int64_t prev = e > 0 ? index_of(keys[e - 1]) : -1;
        for (int64_t r = prev + 1; r <= g; ++r) first[r] = e;
    }
}

// Reads the structure back the way the propagation kernel does and compares every edge with the
// sorted key it was made from, so that a kernel that gathers through it never sees a source or a
// row out of range.  One workgroup per row block; the block's chunk bounds sit in LDS.
__global__ void __launch_bounds__(kBlock) tile_verify_kernel(const uint64_t* __restrict__ keys, int rbits, int vbits,
                                                             int nch, const uint32_t* __restrict__ t_edge,
                                                             const int64_t* __restrict__ first, int64_t N, int64_t M,
                                                             int* __restrict__ bad) {
    extern __shared__ uint32_t bound[];
    const uint64_t rmask = (1ull << rbits) - 1, vmask = (1ull << vbits) - 1;
    for (int64_t rb = blockIdx.x; rb * ((int64_t)1 << rbits) < N; rb += gridDim.x) {
        const int64_t b0 = first[rb * nch], len = first[(rb + 1) * nch] - b0;
        if (b0 < 0 || len < 0 || b0 + len > M || len > 0xFFFFFFFFll) { if (threadIdx.x == 0) *bad = 1; continue; }
        __syncthreads();
        for (int c = threadIdx.x; c <= nch; c += kBlock) bound[c] = (uint32_t)(first[rb * nch + c] - b0);
        __syncthreads();
        for (int64_t p = threadIdx.x; p < len; p += kBlock) {
            const uint64_t k = keys[b0 + p];
            const uint32_t w = t_edge[b0 + p];
            const int c = tile_chunk_of(bound, nch, (uint32_t)p);
            const bool ok = (int64_t)(k >> (vbits + rbits)) == rb && tile_source(w, c) == (uint32_t)((k >> rbits) & vmask) &&
                            (w & kTileRowMask) == (uint32_t)(k & rmask) && (int64_t)tile_source(w, c) < N &&
                            (rb << rbits) + (int64_t)(w & kTileRowMask) < N;
            if (!ok) *bad = 1;
        }
    }
}

// The edges grouped by destination row block and sorted by source inside a block.
static int build_tiles(spp_ctx* ctx, spp_graph* g) {
    hipStream_t st = ctx->stream;
    const int64_t N = g->N, M = g->M;
    const int grid = ctx->num_cu * 8;
    int lds = 0;
    SPP_HIP(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, ctx->device));
    const int nch = (int)((N + ((int64_t)1 << kTileSrcLoBits) - 1) >> kTileSrcLoBits);
    // the fp64 sums of a block and the block's chunk bounds share the LDS of a workgroup
    const size_t bound_bytes = (size_t)(nch + 1) * sizeof(uint32_t);
    const int rbits = (size_t)lds >= (sizeof(double) << kTileRowBits) + bound_bytes + 1024 ? kTileRowBits : kTileRowBits - 1;
    SPP_CHECK((size_t)lds >= (sizeof(double) << rbits) + bound_bytes + 1024, SPP_E_HIP,
              "row blocks: %d bytes of LDS per workgroup do not hold a block's sums and chunk bounds", lds);
    int vbits = 1;
    while (((int64_t)1 << vbits) < N) ++vbits;
    const int64_t nrb = (N + ((int64_t)1 << rbits) - 1) >> rbits;
    int bbits = 1;
    while (((int64_t)1 << bbits) < nrb) ++bbits;
    g->tile_rbits = rbits; g->nrb = nrb; g->nch = nch;
    const int64_t nfirst = nrb * nch + 1;
    SPP_HIP(hipMalloc(&g->tile_first, (size_t)nfirst * sizeof(int64_t)));
    SPP_HIP(hipMalloc(&g->t_edge, (size_t)(M > 0 ? M : 1) * sizeof(uint32_t)));
    fill_i64_kernel<<<grid, kBlock, 0, st>>>(g->tile_first, nfirst, M);
    if (M > 0) {
        uint64_t *ka = nullptr, *kb = nullptr, *sorted = nullptr;
        int* d_bad = nullptr;
        SPP_HIP(hipMalloc(&ka, (size_t)M * sizeof(uint64_t)));
        hipError_t e = hipMalloc(&kb, (size_t)M * sizeof(uint64_t));
        if (e == hipSuccess) e = hipMalloc(&d_bad, sizeof(int));
        if (e != hipSuccess) {
            (void)hipFree(ka); if (kb) (void)hipFree(kb);
            set_error("row blocks: out of device memory for sort keys");
            return SPP_E_OOM;
        }
        tile_keys_kernel<<<grid, kBlock, 0, st>>>(N, g->rowptr, g->col, rbits, vbits, ka);
        int rc = radix_sort_u64(ctx, ka, kb, M, rbits, rbits + vbits + bbits, &sorted);
        if (rc == SPP_OK) {
            int bad = 0;
            tile_lists_kernel<<<grid, kBlock, 0, st>>>(sorted, M, rbits, vbits, nch, g->t_edge, g->tile_first);
            hipError_t e2 = hipMemsetAsync(d_bad, 0, sizeof(int), st);
            if (e2 == hipSuccess) {
                const int vgrid = (int)(nrb < (int64_t)ctx->num_cu * 8 ? nrb : (int64_t)ctx->num_cu * 8);
                tile_verify_kernel<<<vgrid, kBlock, bound_bytes, st>>>(sorted, rbits, vbits, nch, g->t_edge, g->tile_first,
                                                                       N, M, d_bad);
                e2 = hipMemcpyAsync(&bad, d_bad, sizeof(int), hipMemcpyDeviceToHost, st);
            }
            if (e2 == hipSuccess) e2 = hipStreamSynchronize(st);
            if (e2 != hipSuccess) { set_error("row blocks: %s", hipGetErrorString(e2)); rc = SPP_E_HIP; }
            else if (bad) { set_error("row blocks: the structure does not read back as the edges it was built from"); rc = SPP_E_HIP; }
        }
        (void)hipFree(ka); (void)hipFree(kb); (void)hipFree(d_bad);
        SPP_TRY(rc);
    }
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
        int rc = spp::build_tiles(ctx, g);
        if (rc != SPP_OK) { spp_graph_destroy(g); return rc; }
        g->has_in = true;
    }
    *out = g;
    return SPP_OK;
}

extern "C" void spp_graph_destroy(spp_graph* g) {
    if (!g) return;
    if (hipSetDevice(g->device) != hipSuccess) { (void)hipGetLastError(); delete g; return; }   // runtime already shut down
    (void)hipDeviceSynchronize();      // work that still reads the row blocks may be in flight
    if (g->t_edge) (void)hipFree(g->t_edge);
    if (g->tile_first) (void)hipFree(g->tile_first);
    delete g;
}
