// Stable least-significant-digit radix sort of 64-bit keys, 8 bits per pass, used at set-up time:
// to build the transposed edge structure (edge keys packed as (row block of u, source v, row of u
// inside its block), sorted on the block and source bits, which groups the edges by destination
// row block and orders them by source inside a block) and to rank cache candidates and local
// vertices (Sec. 3.2).
//
// A tile is 4096 keys handled by one 256-thread workgroup; wavefront w owns the w-th quarter of
// the tile and walks it in order, 64 keys at a time, so a key's stable rank among equal digits is
// (count of that digit in earlier wavefronts' quarters) + (count earlier in its own quarter) +
// (count in lower lanes of its own 64), the last from ballots.  Keys are then placed in digit
// order in LDS and written out as per-digit runs.
#include "spp_common.h"
#include "spp_device.h"

namespace spp {

constexpr int kTile = 4096;
constexpr int kPerWave = kTile / 4;          // 1024 keys per wavefront
constexpr int kBatches = kPerWave / kWave;   // 16 batches of 64

__global__ void __launch_bounds__(kBlock) radix_hist_kernel(const uint64_t* __restrict__ keys, int64_t n,
                                                            int shift, int64_t ntiles,
                                                            uint32_t* __restrict__ hist) {
    __shared__ uint32_t h[256];
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        h[threadIdx.x] = 0;
        __syncthreads();
        const int64_t base = tile * kTile;
        for (int k = threadIdx.x; k < kTile; k += kBlock) {
            int64_t i = base + k;
            if (i < n) atomicAdd(&h[(uint32_t)(keys[i] >> shift) & 255u], 1u);
        }
        __syncthreads();
        hist[(int64_t)threadIdx.x * ntiles + tile] = h[threadIdx.x];
        __syncthreads();
    }
}

struct HistIn  { const uint32_t* h; __device__ int operator()(int64_t i) const { return (int)h[i]; } };
struct HistOut { uint32_t* h; __device__ void operator()(int64_t i, int ex, int) const { h[i] = (uint32_t)ex; } };
struct NoFin   { __device__ void operator()(int) const {} };

__global__ void __launch_bounds__(kBlock) radix_scatter_kernel(const uint64_t* __restrict__ keys,
                                                               uint64_t* __restrict__ out, int64_t n,
                                                               int shift, int64_t ntiles,
                                                               const uint32_t* __restrict__ offs) {
    __shared__ uint32_t cnt[4][256];
    __shared__ uint32_t dstart[256];
    __shared__ uint32_t gbase[256];
    __shared__ uint64_t sorted[kTile];
    __shared__ int scan_lds[4];
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));

    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        for (int w = 0; w < 4; ++w) cnt[w][threadIdx.x] = 0;
        __syncthreads();

        uint64_t key[kBatches];
        uint16_t rnk[kBatches];
        const int64_t wbase = tile * kTile + (int64_t)wave * kPerWave;
#pragma unroll
        for (int b = 0; b < kBatches; ++b) {
            const int64_t i = wbase + b * kWave + lane;
            const bool valid = i < n;
            const uint64_t k = valid ? keys[i] : 0ull;
            const uint32_t d = (uint32_t)(k >> shift) & 255u;
            uint64_t m = __ballot(valid);
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const bool one = (d >> bit) & 1u;
                const uint64_t bm = __ballot(valid && one);
                m &= one ? bm : ~bm;
            }
            const uint32_t below = (uint32_t)__popcll(m & lt_mask);
            uint32_t prior = 0;
            if (valid) prior = cnt[wave][d];
            if (valid && below == 0) cnt[wave][d] = prior + (uint32_t)__popcll(m);
            key[b] = k;
            rnk[b] = (uint16_t)(prior + below);
        }
        __syncthreads();

        {   // digit totals -> start of each digit's run in the tile, and per-wavefront offsets
            const int d = threadIdx.x;
            const uint32_t c0 = cnt[0][d], c1 = cnt[1][d], c2 = cnt[2][d], c3 = cnt[3][d];
            int total;
            const int ex = block_exclusive_scan((int)(c0 + c1 + c2 + c3), scan_lds, total);
            dstart[d] = (uint32_t)ex;
            cnt[0][d] = (uint32_t)ex;
            cnt[1][d] = (uint32_t)ex + c0;
            cnt[2][d] = (uint32_t)ex + c0 + c1;
            cnt[3][d] = (uint32_t)ex + c0 + c1 + c2;
            gbase[d] = offs[(int64_t)d * ntiles + tile];
        }
        __syncthreads();

#pragma unroll
        for (int b = 0; b < kBatches; ++b) {
            const int64_t i = wbase + b * kWave + lane;
            if (i < n) {
                const uint32_t d = (uint32_t)(key[b] >> shift) & 255u;
                sorted[cnt[wave][d] + rnk[b]] = key[b];
            }
        }
        __syncthreads();

        const int64_t left = n - tile * kTile;
        const int count = left < kTile ? (int)left : kTile;
        for (int k = threadIdx.x; k < count; k += kBlock) {
            const uint64_t v = sorted[k];
            const uint32_t d = (uint32_t)(v >> shift) & 255u;
            out[(uint64_t)gbase[d] + (uint32_t)(k - dstart[d])] = v;
        }
        __syncthreads();
    }
}

int radix_sort_u64(spp_ctx* ctx, uint64_t* keys_a, uint64_t* keys_b, int64_t n, int bit_lo, int bit_hi,
                   uint64_t** result) {
    *result = keys_a;
    if (n <= 1 || bit_hi <= bit_lo) return SPP_OK;
    SPP_CHECK(n < (int64_t)0xFFFFFFFFll, SPP_E_ARG, "radix_sort_u64: %lld keys exceed the 32-bit offset range",
              (long long)n);
    hipStream_t st = ctx->stream;
    const int64_t ntiles = (n + kTile - 1) / kTile;
    const int64_t nhist = 256 * ntiles;
    uint32_t* hist = nullptr;
    int64_t* d_n = nullptr;
    int* partial = nullptr;
    const int scan_grid = 1024;
    SPP_HIP(hipMalloc(&hist, (size_t)nhist * sizeof(uint32_t)));
    hipError_t e1 = hipMalloc(&d_n, sizeof(int64_t));
    hipError_t e2 = hipMalloc(&partial, scan_grid * sizeof(int));
    if (e1 != hipSuccess || e2 != hipSuccess) {
        (void)hipFree(hist); if (d_n) (void)hipFree(d_n); if (partial) (void)hipFree(partial);
        set_error("radix_sort_u64: workspace allocation failed");
        return SPP_E_OOM;
    }
    int rc = SPP_OK;
    hipError_t e = hipMemcpyAsync(d_n, &nhist, sizeof(int64_t), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);      // nhist lives on this stack frame
    const int grid = (int)(ntiles < (int64_t)ctx->num_cu * 8 ? ntiles : (int64_t)ctx->num_cu * 8);
    uint64_t* src = keys_a;
    uint64_t* dst = keys_b;
    for (int shift = bit_lo; shift < bit_hi && e == hipSuccess; shift += 8) {
        radix_hist_kernel<<<grid, kBlock, 0, st>>>(src, n, shift, ntiles, hist);
        grid_scan(st, scan_grid, d_n, HistIn{hist}, HistOut{hist}, NoFin{}, partial);
        radix_scatter_kernel<<<grid, kBlock, 0, st>>>(src, dst, n, shift, ntiles, hist);
        e = hipGetLastError();
        uint64_t* t = src; src = dst; dst = t;
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        set_error("radix_sort_u64: %s", hipGetErrorString(e));
        rc = SPP_E_HIP;
    }
    (void)hipFree(hist); (void)hipFree(d_n); (void)hipFree(partial);
    *result = src;
    return rc;
}

}  // namespace spp
