// Context, error text and timing of the library; see include/spp.h for the contract.
#include "spp_common.h"

#include <new>

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
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&c->h_pinned), 64 * sizeof(int64_t), hipHostMallocDefault);
    for (int i = 0; i < spp::kNumTimers && e == hipSuccess; ++i) {
        e = hipEventCreate(&c->t0[i]);
        if (e == hipSuccess) e = hipEventCreate(&c->t1[i]);
    }
    if (e != hipSuccess) {
        spp::set_error("spp_ctx_create: %s", hipGetErrorString(e));
        spp_ctx_destroy(c);
        return SPP_E_HIP;
    }
    memset(c->h_pinned, 0, 64 * sizeof(int64_t));
    *out = c;
    return SPP_OK;
}

extern "C" void spp_ctx_destroy(spp_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->stream);
    if (c->side) { (void)hipStreamSynchronize(c->side); (void)hipStreamDestroy(c->side); }
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    for (int i = 0; i < spp::kNumTimers; ++i) {
        if (c->t0[i]) (void)hipEventDestroy(c->t0[i]);
        if (c->t1[i]) (void)hipEventDestroy(c->t1[i]);
    }
    if (c->h_pinned) (void)hipHostFree(c->h_pinned);
    c->table.release(); c->flat.release(); c->partials.release();
    c->srcdesc.release(); c->misslist.release(); c->gcount.release();
    c->y0.release(); c->y1.release(); c->tot.release(); c->hubacc.release();
    delete c;
}

extern "C" int spp_ctx_sync(spp_ctx* c) {
    SPP_CHECK(c != nullptr, SPP_E_ARG, "spp_ctx_sync: ctx is null");
    SPP_HIP(hipStreamSynchronize(c->stream));
    SPP_HIP(hipStreamSynchronize(c->side));
    return SPP_OK;
}

extern "C" int spp_ctx_timing(spp_ctx* c, int enable) {
    SPP_CHECK(c != nullptr, SPP_E_ARG, "spp_ctx_timing: ctx is null");
    c->timing = enable ? 1 : 0;
    if (!enable) for (int i = 0; i < spp::kNumTimers; ++i) c->t_valid[i] = false;
    return SPP_OK;
}

extern "C" int spp_ctx_last_times(spp_ctx* c, float* ms_out) {
    SPP_CHECK(c != nullptr && ms_out != nullptr, SPP_E_ARG, "spp_ctx_last_times: null argument");
    for (int i = 0; i < spp::kNumTimers; ++i) {
        ms_out[i] = -1.0f;
        if (!c->t_valid[i]) continue;
        float ms = 0.f;
        hipError_t e = hipEventElapsedTime(&ms, c->t0[i], c->t1[i]);
        if (e == hipSuccess) ms_out[i] = ms;
    }
    return SPP_OK;
}
