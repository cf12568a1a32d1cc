// Device-side building blocks shared by the kernels: wavefront (64-lane) scans, a three-launch
// grid scan whose length is read on the device, the open-addressing id table, Philox-4x32-10.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spp {

constexpr int kBlock = 256;            // threads per workgroup: 4 wavefronts of 64 lanes
constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Prefix sums are formed modulo 2^32 (counts up to 2^32 - 1 pass through int unchanged).
__device__ __forceinline__ int uadd(int a, int b) { return (int)((unsigned)a + (unsigned)b); }

// Inclusive scan over the 64 lanes of a wavefront.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        int t = __shfl_up(v, off, kWave);
        if (lane >= off) v = uadd(v, t);
    }
    return v;
}

// Exclusive scan over a 256-thread workgroup; returns the exclusive prefix of `v` and the
// workgroup total in `total`.  `lds` needs 4 ints.  Ends with a barrier, so it can be called in a loop.
__device__ __forceinline__ int block_exclusive_scan(int v, int* lds, int& total) {
    const int wave = threadIdx.x >> 6, lane = lane_id();
    int inc = wave_inclusive_scan(v);
    if (lane == kWave - 1) lds[wave] = inc;
    __syncthreads();
    int w0 = lds[0], w1 = lds[1], w2 = lds[2], w3 = lds[3];
    int base = uadd(uadd(wave > 0 ? w0 : 0, wave > 1 ? w1 : 0), wave > 2 ? w2 : 0);
    total = uadd(uadd(w0, w1), uadd(w2, w3));
    __syncthreads();
    return (int)((unsigned)base + (unsigned)inc - (unsigned)v);
}

__device__ __forceinline__ int block_reduce_sum(int v, int* lds) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v = uadd(v, __shfl_down(v, off, kWave));
    if (lane_id() == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = uadd(uadd(lds[0], lds[1]), uadd(lds[2], lds[3]));
    __syncthreads();
    return t;
}

// ---------------------------------------------------------------------------------------------
// Grid scan in three launches over i in [0, n), n read from device memory (so no host round trip
// is needed between dependent steps).  Work is cut into `gridDim.x` contiguous ranges.
//   In:  int operator()(int64_t i) const            value of element i
//   Out: void operator()(int64_t i, int ex, int v)  receives the exclusive prefix
//   Fin: void operator()(int total) const           called once by one thread
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void scan_range(int64_t n, int64_t& begin, int64_t& end) {
    int64_t per = (n + gridDim.x - 1) / gridDim.x;
    per = (per + kBlock - 1) / kBlock * kBlock;
    begin = (int64_t)blockIdx.x * per;
    end = begin + per < n ? begin + per : n;
    if (begin > n) begin = n;
}

template <class In>
__global__ void __launch_bounds__(kBlock) scan_reduce_kernel(const int64_t* n_ptr, In in, int* partial) {
    __shared__ int lds[4];
    int64_t b, e;
    scan_range(*n_ptr, b, e);
    int acc = 0;
    for (int64_t i = b + threadIdx.x; i < e; i += kBlock) acc = uadd(acc, in(i));
    int t = block_reduce_sum(acc, lds);
    if (threadIdx.x == 0) partial[blockIdx.x] = t;
}

template <class Fin>
__global__ void __launch_bounds__(kBlock) scan_partials_kernel(int* partial, int nparts, Fin fin) {
    __shared__ int lds[4];
    int carry = 0;
    for (int base = 0; base < nparts; base += kBlock) {
        int i = base + threadIdx.x;
        int v = i < nparts ? partial[i] : 0;
        int total;
        int ex = block_exclusive_scan(v, lds, total);
        if (i < nparts) partial[i] = uadd(carry, ex);
        carry = uadd(carry, total);
    }
    if (threadIdx.x == 0) fin(carry);
}

template <class In, class Out>
__global__ void __launch_bounds__(kBlock) scan_write_kernel(const int64_t* n_ptr, In in, Out out,
                                                            const int* partial) {
    __shared__ int lds[4];
    int64_t b, e;
    scan_range(*n_ptr, b, e);
    int carry = partial[blockIdx.x];
    for (int64_t base = b; base < e; base += kBlock) {
        int64_t i = base + threadIdx.x;
        int v = i < e ? in(i) : 0;
        int total;
        int ex = block_exclusive_scan(v, lds, total);
        if (i < e) out(i, uadd(carry, ex), v);
        carry = uadd(carry, total);
    }
}

template <class In, class Out, class Fin>
inline void grid_scan(hipStream_t st, int grid, const int64_t* n_ptr, In in, Out out, Fin fin, int* partial) {
    scan_reduce_kernel<In><<<grid, kBlock, 0, st>>>(n_ptr, in, partial);
    scan_partials_kernel<Fin><<<1, kBlock, 0, st>>>(partial, grid, fin);
    scan_write_kernel<In, Out><<<grid, kBlock, 0, st>>>(n_ptr, in, out, partial);
}

// The same scan for several independent sequences at once: blockIdx.y names the sequence ("batch") j.
//   In:  int64_t n(int j) const (length, read on the device); int operator()(int j, int64_t i) const
//   Out: void operator()(int j, int64_t i, int ex, int v) const
//   Fin: void operator()(int j, int total) const
// `partial` holds gridDim.x ints per sequence.
template <class In>
__global__ void __launch_bounds__(kBlock) bscan_reduce_kernel(In in, int* partial) {
    __shared__ int lds[4];
    const int j = blockIdx.y;
    int64_t b, e;
    scan_range(in.n(j), b, e);
    int acc = 0;
    for (int64_t i = b + threadIdx.x; i < e; i += kBlock) acc = uadd(acc, in(j, i));
    int t = block_reduce_sum(acc, lds);
    if (threadIdx.x == 0) partial[(int64_t)j * gridDim.x + blockIdx.x] = t;
}

template <class Fin>
__global__ void __launch_bounds__(kBlock) bscan_partials_kernel(int* partial, int nparts, Fin fin) {
    __shared__ int lds[4];
    const int j = blockIdx.x;                       // one workgroup per sequence
    int* p = partial + (int64_t)j * nparts;
    int carry = 0;
    for (int base = 0; base < nparts; base += kBlock) {
        int i = base + threadIdx.x;
        int v = i < nparts ? p[i] : 0;
        int total;
        int ex = block_exclusive_scan(v, lds, total);
        if (i < nparts) p[i] = uadd(carry, ex);
        carry = uadd(carry, total);
    }
    if (threadIdx.x == 0) fin(j, carry);
}

template <class In, class Out>
__global__ void __launch_bounds__(kBlock) bscan_write_kernel(In in, Out out, const int* partial) {
    __shared__ int lds[4];
    const int j = blockIdx.y;
    int64_t b, e;
    scan_range(in.n(j), b, e);
    int carry = partial[(int64_t)j * gridDim.x + blockIdx.x];
    for (int64_t base = b; base < e; base += kBlock) {
        int64_t i = base + threadIdx.x;
        int v = i < e ? in(j, i) : 0;
        int total;
        int ex = block_exclusive_scan(v, lds, total);
        if (i < e) out(j, i, uadd(carry, ex), v);
        carry = uadd(carry, total);
    }
}

template <class In, class Out, class Fin>
inline void grid_scan_batched(hipStream_t st, int grid, int nbatch, In in, Out out, Fin fin, int* partial) {
    bscan_reduce_kernel<In><<<dim3(grid, nbatch), kBlock, 0, st>>>(in, partial);
    bscan_partials_kernel<Fin><<<nbatch, kBlock, 0, st>>>(partial, grid, fin);
    bscan_write_kernel<In, Out><<<dim3(grid, nbatch), kBlock, 0, st>>>(in, out, partial);
}

// ---------------------------------------------------------------------------------------------
// Open-addressing table of 64-bit entries (key << 32 | value), empty = all ones, linear probing.
// The capacity is a power of two at least twice the number of keys, so probes end.
// ---------------------------------------------------------------------------------------------
constexpr uint64_t kEmpty = ~0ull;

__device__ __forceinline__ uint32_t table_hash(uint32_t key, int shift) {
    return (key * 0x9E3779B1u) >> shift;         // top log2(capacity) bits of a Fibonacci product
}

// Keeps, per key, the smallest value ever offered; returns the slot that holds the key.
__device__ __forceinline__ uint32_t table_insert_min(unsigned long long* tab, uint32_t mask, int shift,
                                                     uint32_t key, uint32_t value) {
    const unsigned long long want = ((unsigned long long)key << 32) | value;
    uint32_t h = table_hash(key, shift);
    for (;;) {
        unsigned long long cur = __hip_atomic_load(&tab[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (cur == kEmpty) {
            unsigned long long old = atomicCAS(&tab[h], (unsigned long long)kEmpty, want);
            if (old == kEmpty) return h;
            cur = old;
        }
        if ((uint32_t)(cur >> 32) == key) {
            if (want < cur) atomicMin(&tab[h], want);
            return h;
        }
        h = (h + 1) & mask;
    }
}

// Returns the slot index of `key`, or -1; `value` receives the stored value.
__device__ __forceinline__ int64_t table_find(const unsigned long long* tab, uint32_t mask, int shift,
                                              uint32_t key, uint32_t& value) {
    uint32_t h = table_hash(key, shift);
    for (;;) {
        unsigned long long cur = __hip_atomic_load(&tab[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (cur == kEmpty) return -1;
        if ((uint32_t)(cur >> 32) == key) { value = (uint32_t)cur; return (int64_t)h; }
        h = (h + 1) & mask;
    }
}

// ---------------------------------------------------------------------------------------------
// Philox-4x32 with 10 rounds (Salmon et al., SC'11), from the published round function:
// two 32x32->64 multiplies per round, key bumped by the Weyl constants between rounds.
// ---------------------------------------------------------------------------------------------
struct Philox4 { uint32_t w[4]; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    Philox4 out;
    out.w[0] = c0; out.w[1] = c1; out.w[2] = c2; out.w[3] = c3;
    return out;
}

// The draw for (seed, batch, hop, vertex, slot).
__device__ __forceinline__ uint32_t rand32(uint64_t seed, uint32_t batch_lo, uint32_t hop, uint32_t vertex,
                                           uint32_t slot) {
    Philox4 p = philox4x32_10(vertex, slot >> 2, hop, batch_lo, (uint32_t)seed, (uint32_t)(seed >> 32));
    const uint32_t s = slot & 3u;
    return s == 0 ? p.w[0] : s == 1 ? p.w[1] : s == 2 ? p.w[2] : p.w[3];
}

}  // namespace spp
