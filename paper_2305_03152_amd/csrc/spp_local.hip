// VIP-ordered local storage (Sec. 3.2, paragraph on host-to-device transfer reduction; Sec. 4.1):
// rank the partition's own vertices by decreasing score, keep the rows of the first
// floor(beta * (hi-lo)) of that order in device memory (in rank order), leave the others in the
// caller's host array.  The paper renumbers the vertices so that the device-resident ones are a
// prefix of the partition's id range; here ids stay as they are and an int32 rank per local vertex
// plays the part of the renumbering (4 bytes per local vertex, read once per gathered local id).
//
// Keys are (~score bits) << 32 | local index in ascending index order, stably radix-sorted on the
// score bits: floats >= 0 order like their bit patterns, the complement turns that into descending
// score, and stability keeps ascending id among equal scores.  Scores that are not positive
// (negative, zero, not a number) are replaced by 0.
#include "spp_common.h"
#include "spp_device.h"
#include "spp_rowcopy.h"

#include <math.h>
#include <new>

namespace spp {

__global__ void __launch_bounds__(kBlock) local_keys_kernel(const float* __restrict__ score, int64_t lo, int64_t n,
                                                            uint64_t* __restrict__ keys) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        const float s = score[lo + i];
        const float c = s > 0.0f ? s : 0.0f;              // false for NaN too
        keys[i] = ((uint64_t)(~__float_as_uint(c)) << 32) | (uint32_t)i;
    }
}

__global__ void __launch_bounds__(kBlock) local_rank_kernel(const uint64_t* __restrict__ sorted, int64_t n,
                                                            int64_t n_rows, int32_t* __restrict__ rank,
                                                            int64_t* __restrict__ rowidx) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x; r < n; r += stride) {
        const uint32_t i = (uint32_t)sorted[r];
        rank[i] = (int32_t)r;
        if (r < n_rows) rowidx[r] = (int64_t)i;
    }
}

__global__ void __launch_bounds__(kBlock) local_lookup_kernel(const int32_t* __restrict__ rank, int64_t lo, int64_t hi,
                                                              const int32_t* __restrict__ ids, int64_t n,
                                                              int32_t* __restrict__ out) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        const int64_t g = ids[i];
        out[i] = (g >= lo && g < hi) ? rank[g - lo] : -1;
    }
}

}  // namespace spp

extern "C" int spp_build_local_store(spp_ctx* ctx, const float* d_score, int64_t N, int64_t lo, int64_t hi,
                                     double beta, const void* local_rows, int32_t D, int32_t elem_bytes,
                                     int64_t* n_device_rows, spp_local_store** out) {
    using namespace spp;
    SPP_CHECK(ctx && d_score && n_device_rows && out, SPP_E_ARG, "spp_build_local_store: null argument");
    *out = nullptr; *n_device_rows = 0;
    SPP_CHECK(N > 0 && N <= 0x7FFFFFFFll && lo >= 0 && lo <= hi && hi <= N, SPP_E_ARG,
              "spp_build_local_store: range [%lld, %lld) of N = %lld", (long long)lo, (long long)hi, (long long)N);
    SPP_CHECK(beta >= 0.0 && beta == beta, SPP_E_ARG, "spp_build_local_store: beta = %g", beta);
    SPP_CHECK(D >= 1 && elem_bytes >= 1 && ((int64_t)D * elem_bytes) % 2 == 0, SPP_E_ARG,
              "spp_build_local_store: D = %d, elem_bytes = %d", D, elem_bytes);
    const int64_t n = hi - lo;
    SPP_CHECK(n == 0 || local_rows, SPP_E_ARG, "spp_build_local_store: local_rows is null");
    double cd = floor(beta * (double)n);
    if (cd > (double)n) cd = (double)n;
    const int64_t keep = (int64_t)cd;
    SPP_HIP(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;

    spp_local_store* s = new (std::nothrow) spp_local_store();
    SPP_CHECK(s != nullptr, SPP_E_OOM, "spp_build_local_store: out of host memory");
    s->device = ctx->device; s->N = N; s->lo = lo; s->hi = hi; s->row_bytes = (int64_t)D * elem_bytes;

    int rc = SPP_OK;
    uint64_t *ka = nullptr, *kb = nullptr, *sorted = nullptr;
    int64_t* rowidx = nullptr;
    do {
        if (n == 0) break;
        rc = device_view(local_rows, &s->host_rows);
        if (rc != SPP_OK) break;
        if (hipMalloc(&ka, (size_t)n * sizeof(uint64_t)) != hipSuccess ||
            hipMalloc(&kb, (size_t)n * sizeof(uint64_t)) != hipSuccess ||
            hipMalloc(&s->rank, (size_t)n * sizeof(int32_t)) != hipSuccess ||
            hipMalloc(&rowidx, (size_t)(keep > 0 ? keep : 1) * sizeof(int64_t)) != hipSuccess) {
            set_error("spp_build_local_store: out of device memory for %lld local vertices", (long long)n);
            rc = SPP_E_OOM; break;
        }
        const int64_t need = (n + kBlock - 1) / kBlock;
        const int grid = (int)(need < (int64_t)ctx->num_cu * 8 ? need : (int64_t)ctx->num_cu * 8);
        local_keys_kernel<<<grid, kBlock, 0, st>>>(d_score, lo, n, ka);
        rc = radix_sort_u64(ctx, ka, kb, n, 32, 64, &sorted);
        if (rc != SPP_OK) break;
        local_rank_kernel<<<grid, kBlock, 0, st>>>(sorted, n, keep, s->rank, rowidx);
        if (keep > 0) {
            if (hipMalloc(&s->rows, (size_t)keep * (size_t)s->row_bytes) != hipSuccess) {
                set_error("spp_build_local_store: out of device memory for %lld local rows", (long long)keep);
                rc = SPP_E_OOM; break;
            }
            rc = copy_rows_indexed(st, local_rows, rowidx, keep, s->row_bytes, s->rows, ctx->num_cu);
            if (rc != SPP_OK) break;
        }
        if (hipStreamSynchronize(st) != hipSuccess) {
            set_error("spp_build_local_store: %s", hipGetErrorString(hipGetLastError())); rc = SPP_E_HIP; break;
        }
    } while (0);

    if (ka) (void)hipFree(ka);
    if (kb) (void)hipFree(kb);
    if (rowidx) (void)hipFree(rowidx);
    if (rc != SPP_OK) { spp_local_store_destroy(s); return rc; }
    s->n_rows = n == 0 ? 0 : keep; s->limit = s->n_rows;
    *n_device_rows = s->n_rows;
    *out = s;
    return SPP_OK;
}

extern "C" void spp_local_store_destroy(spp_local_store* s) {
    if (!s) return;
    if (hipSetDevice(s->device) != hipSuccess) { (void)hipGetLastError(); delete s; return; }   // runtime already shut down
    (void)hipDeviceSynchronize();      // a gather that still reads the store may be in flight
    if (s->rank) (void)hipFree(s->rank);
    if (s->rows) (void)hipFree(s->rows);
    delete s;
}

extern "C" int spp_local_store_set_limit(spp_local_store* s, int64_t n_rows) {
    SPP_CHECK(s, SPP_E_ARG, "spp_local_store_set_limit: store is null");
    SPP_CHECK(n_rows <= s->n_rows, SPP_E_ARG, "spp_local_store_set_limit: %lld rows asked, %lld built",
              (long long)n_rows, (long long)s->n_rows);
    s->limit = n_rows < 0 ? s->n_rows : n_rows;
    return SPP_OK;
}

extern "C" int spp_local_store_rank(spp_ctx* ctx, const spp_local_store* s, const int32_t* d_ids, int64_t n,
                                    int32_t* d_rank_out) {
    using namespace spp;
    SPP_CHECK(ctx && s && (n == 0 || (d_ids && d_rank_out)), SPP_E_ARG, "spp_local_store_rank: null argument");
    if (n == 0) return SPP_OK;
    SPP_HIP(hipSetDevice(ctx->device));
    const int64_t need = (n + kBlock - 1) / kBlock;
    const int grid = (int)(need < (int64_t)ctx->num_cu * 8 ? need : (int64_t)ctx->num_cu * 8);
    // an empty partition has no rank array: the range test fails for every id
    local_lookup_kernel<<<grid, kBlock, 0, ctx->stream>>>(s->rank, s->lo, s->hi, d_ids, n, d_rank_out);
    SPP_HIP(hipGetLastError());
    return SPP_OK;
}
