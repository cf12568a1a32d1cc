// Context, error text and timing of the library; see include/spp.h for the contract.
#include "spp_common.h"
#include <cstdlib>

#include <algorithm>
#include <new>
#include <vector>

namespace spp {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

}  // namespace spp

extern "C" const char* spp_last_error(void) { return spp::g_err; }

extern "C" int spp_ctx_create(spp_ctx** out, int device, void* hip_stream) {
    SPP_CHECK(out != nullptr, SPP_E_ARG, "spp_ctx_create: out is null");
    *out = nullptr;
    int ndev = 0;
    SPP_HIP(hipGetDeviceCount(&ndev));
    SPP_CHECK(device >= 0 && device < ndev, SPP_E_ARG, "spp_ctx_create: device %d of %d", device, ndev);
    SPP_HIP(hipSetDevice(device));
    void* fixed_ws = nullptr;
    SPP_TRY(spp::static_scratch(device, &fixed_ws));      // this device's address of the allocation-free gather's workspace
    spp_ctx* c = new (std::nothrow) spp_ctx();
    SPP_CHECK(c != nullptr, SPP_E_OOM, "spp_ctx_create: out of host memory");
    c->device = device;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) == hipSuccess && prop.multiProcessorCount > 0)
        c->num_cu = prop.multiProcessorCount;
    // default priority on purpose: streams of mixed priority are not used anywhere in this library
    hipError_t e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_join[0], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_join[1], hipEventDisableTiming);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&c->h_pinned), 8192 * sizeof(int64_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->totals), 16 * sizeof(int64_t));
    if (e == hipSuccess) e = hipMemset(c->totals, 0, 16 * sizeof(int64_t));
    if (e != hipSuccess) {
        spp::set_error("spp_ctx_create: %s", hipGetErrorString(e));
        spp_ctx_destroy(c);
        return SPP_E_HIP;
    }
    memset(c->h_pinned, 0, 8192 * sizeof(int64_t));
    *out = c;
    return SPP_OK;
}

extern "C" void spp_ctx_destroy(spp_ctx* c) {
    if (!c) return;
    // Once the HIP runtime has shut down (a destroy that reaches here during process exit) nothing is
    // left to release on the device, and its handles must not be touched.
    if (hipSetDevice(c->device) != hipSuccess) { (void)hipGetLastError(); delete c; return; }
    (void)hipStreamSynchronize(c->stream);
    if (c->side) { (void)hipStreamSynchronize(c->side); (void)hipStreamDestroy(c->side); }
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    for (hipEvent_t e : c->ev_join) if (e) (void)hipEventDestroy(e);
    for (auto& sp : c->spans) { (void)hipEventDestroy(sp.t0); (void)hipEventDestroy(sp.t1); }
    for (hipEvent_t e : c->ev_free) (void)hipEventDestroy(e);
    if (c->h_pinned) (void)hipHostFree(c->h_pinned);
    if (c->totals) (void)hipFree(c->totals);
    c->table.release(); c->flat.release(); c->nodeinfo.release(); c->slots.release(); c->partials.release();
    c->btab.release(); free(c->btab_mirror);
    c->gtable.release(); c->gfirst.release();
    for (int k = 0; k < 2; ++k) { c->srcdesc[k].release(); c->misslist[k].release(); c->gcount[k].release(); c->hititems[k].release(); }
    c->y0.release(); c->y1.release(); c->tot.release(); c->acc.release(); c->frontier.release(); c->bins.release(); c->xvals.release();
    delete c;
}

extern "C" int spp_ctx_sync(spp_ctx* c) {
    SPP_CHECK(c != nullptr, SPP_E_ARG, "spp_ctx_sync: ctx is null");
    SPP_TRY(spp_gather_join(c));          // a gather left unjoined still owes its shared rows
    SPP_HIP(hipStreamSynchronize(c->stream));
    SPP_HIP(hipStreamSynchronize(c->side));
    return SPP_OK;
}

static void recycle_spans(spp_ctx* c) {
    for (auto& sp : c->spans) { c->ev_free.push_back(sp.t0); c->ev_free.push_back(sp.t1); }
    c->spans.clear();
}

extern "C" int spp_ctx_timing(spp_ctx* c, int enable) {
    SPP_CHECK(c != nullptr, SPP_E_ARG, "spp_ctx_timing: ctx is null");
    SPP_TRY(spp_ctx_sync(c));
    recycle_spans(c);
    c->timing = enable ? 1 : 0;
    return SPP_OK;
}

extern "C" int spp_ctx_time_stats(spp_ctx* c, float* sum_ms, int64_t* count, float* min_ms, float* median_ms) {
    SPP_CHECK(c != nullptr, SPP_E_ARG, "spp_ctx_time_stats: ctx is null");
    SPP_TRY(spp_ctx_sync(c));
    std::vector<float> pieces[spp::kNumTimers];
    for (auto& sp : c->spans) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sp.t0, sp.t1) == hipSuccess && sp.idx >= 0 && sp.idx < spp::kNumTimers)
            pieces[sp.idx].push_back(ms);
    }
    for (int i = 0; i < spp::kNumTimers; ++i) {
        std::vector<float>& v = pieces[i];
        std::sort(v.begin(), v.end());
        float sum = 0.f;
        for (float x : v) sum += x;
        if (sum_ms) sum_ms[i] = sum;
        if (count) count[i] = (int64_t)v.size();
        if (min_ms) min_ms[i] = v.empty() ? 0.f : v.front();
        if (median_ms) median_ms[i] = v.empty() ? 0.f : 0.5f * (v[(v.size() - 1) / 2] + v[v.size() / 2]);
    }
    recycle_spans(c);
    return SPP_OK;
}

extern "C" int spp_ctx_times(spp_ctx* c, float* sum_ms, int64_t* count) {
    SPP_CHECK(c != nullptr && sum_ms != nullptr && count != nullptr, SPP_E_ARG, "spp_ctx_times: null argument");
    return spp_ctx_time_stats(c, sum_ms, count, nullptr, nullptr);
}

extern "C" int spp_ctx_totals(spp_ctx* c, int64_t* out, int reset) {
    SPP_CHECK(c != nullptr && out != nullptr, SPP_E_ARG, "spp_ctx_totals: null argument");
    SPP_TRY(spp_ctx_sync(c));
    SPP_HIP(hipMemcpy(out, c->totals, 16 * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (reset) SPP_HIP(hipMemset(c->totals, 0, 16 * sizeof(int64_t)));
    return SPP_OK;
}

// ---- plain streaming kernels: what the part reaches by direction, for reading rooflines -------
namespace spp {
typedef uint32_t probe_vec __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(512) stream_read_kernel(const probe_vec* __restrict__ p, int64_t nvec, uint32_t* sink) {
    const int64_t stride = (int64_t)gridDim.x * 512;
    int64_t i = (int64_t)blockIdx.x * 512 + threadIdx.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < nvec; i += 4 * stride) {
        probe_vec v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(p + i + u * stride);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < nvec; i += stride) { const probe_vec v = __builtin_nontemporal_load(p + i); acc ^= v.x ^ v.y ^ v.z ^ v.w; }
    if (acc == 0x9E3779B9u) *sink = acc;            // keeps the loads alive; practically never taken
}
// one vector per lane, one tile per workgroup: the shape that copies fastest on this part
__global__ void __launch_bounds__(256) stream_copy_kernel(const probe_vec* __restrict__ s, probe_vec* __restrict__ d, int64_t nvec) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < nvec) __builtin_nontemporal_store(s[i], d + i);
}
__global__ void __launch_bounds__(256) stream_write_kernel(probe_vec* __restrict__ d, int64_t nvec) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const probe_vec v = {(uint32_t)i, 1u, 2u, 3u};
    if (i < nvec) __builtin_nontemporal_store(v, d + i);
}
}  // namespace spp

extern "C" int spp_stream_rates(spp_ctx* c, const void* d_a, void* d_b, int64_t bytes, int32_t reps, float* out_gbps) {
    using namespace spp;
    SPP_CHECK(c && d_a && d_b && out_gbps, SPP_E_ARG, "spp_stream_rates: null argument");
    SPP_CHECK(bytes >= 16 && bytes % 16 == 0 && bytes / 16 / 256 < 0x7FFFFFFFll && reps >= 1 && reps <= 1000, SPP_E_ARG,
              "spp_stream_rates: bytes = %lld (a multiple of 16), reps = %d (1 .. 1000)", (long long)bytes, reps);
    SPP_CHECK((((uintptr_t)d_a | (uintptr_t)d_b) & 15) == 0, SPP_E_ARG, "spp_stream_rates: buffers must be 16-byte aligned");
    SPP_HIP(hipSetDevice(c->device));
    hipStream_t st = c->stream;
    const int64_t nvec = bytes / 16;
    const unsigned tiles = (unsigned)((nvec + 255) / 256);
    const probe_vec* a = static_cast<const probe_vec*>(d_a);
    probe_vec* b = static_cast<probe_vec*>(d_b);
    uint32_t* sink = reinterpret_cast<uint32_t*>(c->totals + 15);       // an unused slot of the running sums
    hipEvent_t e0 = c->take_event(), e1 = c->take_event();
    SPP_CHECK(e0 && e1, SPP_E_HIP, "spp_stream_rates: no events");
    for (int k = 0; k < 3; ++k) {
        const double moved = (k == 1 ? 2.0 : 1.0) * (double)bytes * reps;
        for (int r = -1; r < reps; ++r) {                                // one untimed pass first
            if (r == 0) SPP_HIP(hipEventRecord(e0, st));
            if (k == 0) stream_read_kernel<<<c->num_cu * 64, 512, 0, st>>>(a, nvec, sink);
            else if (k == 1) stream_copy_kernel<<<tiles, 256, 0, st>>>(a, b, nvec);
            else stream_write_kernel<<<tiles, 256, 0, st>>>(b, nvec);
        }
        SPP_HIP(hipEventRecord(e1, st));
        SPP_HIP(hipEventSynchronize(e1));
        float ms = 0.f;
        SPP_HIP(hipEventElapsedTime(&ms, e0, e1));
        out_gbps[k] = ms > 0.f ? (float)(moved / (ms * 1e-3) / 1e9) : 0.f;
    }
    c->ev_free.push_back(e0); c->ev_free.push_back(e1);
    SPP_HIP(hipGetLastError());
    return SPP_OK;
}

extern "C" int spp_vip_last_hops(spp_ctx* c, int32_t* pushed, int64_t* frontier_edges, int32_t L) {
    SPP_CHECK(c != nullptr && L >= 0 && L <= SPP_MAX_L, SPP_E_ARG, "spp_vip_last_hops: bad argument");
    for (int h = 0; h < L; ++h) {
        if (pushed) pushed[h] = c->vip_pushed[h];
        if (frontier_edges) frontier_edges[h] = c->vip_frontier_edges[h];
    }
    return SPP_OK;
}
