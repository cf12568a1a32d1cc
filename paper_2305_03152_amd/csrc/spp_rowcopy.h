// Row-copy kernels shared by the gather and the cache fill.  A row of `row_bytes` bytes is cut
// into vectors of V bytes (V = 16 when sizes and addresses allow: one 128-bit load and store per
// lane); the output is walked as one flat array of vectors, so stores are fully coalesced and
// every lane is busy whatever the row size, while loads are coalesced within a row.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spp_device.h"

namespace spp {

template <int V> struct VecOf;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <> struct VecOf<16> { typedef u32x4 type; };
template <> struct VecOf<8>  { typedef u32x2 type; };
template <> struct VecOf<4>  { typedef uint32_t type; };
template <> struct VecOf<2>  { typedef uint16_t type; };

// Source descriptor of an output row: tag in the top two bits, row index in the store below.
constexpr int kTagLocal = 0, kTagCache = 1, kTagMiss = 2, kTagSkip = 3;
__device__ __host__ __forceinline__ int64_t make_desc(int tag, int64_t row) { return ((int64_t)tag << 62) | row; }
__device__ __forceinline__ int desc_tag(int64_t d) { return (int)(((uint64_t)d) >> 62); }
__device__ __forceinline__ int64_t desc_row(int64_t d) { return d & ((1ll << 62) - 1); }

template <int V>
__device__ __forceinline__ typename VecOf<V>::type load_stream(const void* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const typename VecOf<V>::type*>(p));
}
template <int V>
__device__ __forceinline__ void store_stream(void* p, typename VecOf<V>::type v) {
    __builtin_nontemporal_store(v, reinterpret_cast<typename VecOf<V>::type*>(p));
}

constexpr int kCopyUnroll = 4;

// Hit path: out[i,:] from the local shard or the cache, for the rows tagged so; others untouched.
// n_ptr (device) overrides n when not null.  vpr = vectors per row.
template <int V>
__global__ void __launch_bounds__(kBlock) gather_hit_kernel(const int64_t* __restrict__ desc, int64_t n,
                                                            const int64_t* __restrict__ n_ptr,
                                                            const char* __restrict__ local,
                                                            const char* __restrict__ cache, uint32_t vpr,
                                                            char* __restrict__ out) {
    typedef typename VecOf<V>::type vec_t;
    if (n_ptr) n = *n_ptr;
    const uint64_t total = (uint64_t)n * vpr;
    const bool small = total <= 0xFFFFFFFFull;          // 32-bit division is far cheaper
    const uint64_t span = (uint64_t)kBlock * kCopyUnroll;
    for (uint64_t base = (uint64_t)blockIdx.x * span; base < total; base += (uint64_t)gridDim.x * span) {
        vec_t v[kCopyUnroll];
        bool ok[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const uint64_t c = base + (uint64_t)u * kBlock + threadIdx.x;
            ok[u] = false;
            if (c < total) {
                const uint64_t i = small ? (uint64_t)((uint32_t)c / vpr) : c / vpr;
                const uint32_t k = (uint32_t)(c - i * vpr);
                const int64_t d = desc[i];
                const int tag = desc_tag(d);
                if (tag <= kTagCache) {
                    const char* src = (tag == kTagLocal ? local : cache) + (desc_row(d) * vpr + k) * (int64_t)V;
                    v[u] = load_stream<V>(src);
                    ok[u] = true;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const uint64_t c = base + (uint64_t)u * kBlock + threadIdx.x;
            if (ok[u]) store_stream<V>(out + c * (uint64_t)V, v[u]);
        }
    }
}

// Indexed rows from one store (pinned host memory over PCIe, or device memory):
//   out[dst(m),:] = src[row(m),:], m < count (read on the device when count_ptr is given).
//   list == null: dst(m) = m, row(m) = rowidx[m]            (cache fill)
//   list != null: dst(m) = list[m], row(m) = desc_row(desc[list[m]])   (miss path)
template <int V>
__global__ void __launch_bounds__(kBlock) rows_indexed_kernel(const char* __restrict__ src,
                                                              const int64_t* __restrict__ rowidx_or_desc,
                                                              const int32_t* __restrict__ list, int64_t count,
                                                              const int64_t* __restrict__ count_ptr, uint32_t vpr,
                                                              char* __restrict__ out) {
    typedef typename VecOf<V>::type vec_t;
    if (count_ptr) count = *count_ptr;
    const uint64_t total = (uint64_t)count * vpr;
    const bool small = total <= 0xFFFFFFFFull;
    const uint64_t span = (uint64_t)kBlock * kCopyUnroll;
    for (uint64_t base = (uint64_t)blockIdx.x * span; base < total; base += (uint64_t)gridDim.x * span) {
        vec_t v[kCopyUnroll];
        uint64_t dst[kCopyUnroll];
        bool ok[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const uint64_t c = base + (uint64_t)u * kBlock + threadIdx.x;
            ok[u] = c < total;
            if (ok[u]) {
                const uint64_t m = small ? (uint64_t)((uint32_t)c / vpr) : c / vpr;
                const uint32_t k = (uint32_t)(c - m * vpr);
                int64_t row, orow;
                if (list) { orow = list[m]; row = desc_row(rowidx_or_desc[orow]); }
                else      { orow = (int64_t)m; row = rowidx_or_desc[m]; }
                v[u] = load_stream<V>(src + ((uint64_t)row * vpr + k) * (uint64_t)V);
                dst[u] = ((uint64_t)orow * vpr + k) * (uint64_t)V;
            }
        }
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (ok[u]) store_stream<V>(out + dst[u], v[u]);
    }
}

// Widest vector that divides the row size and is honoured by every address.
inline int pick_vec(int64_t row_bytes, const void* a, const void* b, const void* c, const void* d) {
    uintptr_t bits = (uintptr_t)row_bytes | (uintptr_t)a | (uintptr_t)b | (uintptr_t)c | (uintptr_t)d;
    if ((bits & 15) == 0) return 16;
    if ((bits & 7) == 0) return 8;
    if ((bits & 3) == 0) return 4;
    return 2;
}

}  // namespace spp
