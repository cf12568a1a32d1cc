// Device-side building blocks shared by the kernels: wavefront (64-lane) scans, grid scans whose
// length is read on the device (three launches; two for several sequences at once), the
// open-addressing id table, Philox-4x32-10.
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
__device__ __forceinline__ void scan_range(int64_t n, unsigned block, int64_t& begin, int64_t& end) {
    int64_t per = (n + gridDim.x - 1) / gridDim.x;
    per = (per + kBlock - 1) / kBlock * kBlock;
    begin = (int64_t)block * per;
    end = begin + per < n ? begin + per : n;
    if (begin > n) begin = n;
}
__device__ __forceinline__ void scan_range(int64_t n, int64_t& begin, int64_t& end) { scan_range(n, blockIdx.x, begin, end); }

// Which sequence ("batch") and which of its gridDim.x workgroups this workgroup is, in a launch of
// gridDim.x x gridDim.y workgroups over gridDim.y independent sequences.  Workgroups are handed to
// the eight XCDs in turn by their linear index, and each XCD has an L2 of its own, so the mapping
// keeps all workgroups of a sequence on one XCD when the counts allow it (a multiple of 8 sequences,
// or 1/2/4 sequences with gridDim.x a multiple of 8): data that only this sequence touches (its id
// table) then stays in one L2 instead of moving between eight.  Any other shape uses (x, y) as
// given.  Only speed depends on where workgroups land; every shape is a bijection.
struct BatchBlock { int j; unsigned x; };
__device__ __forceinline__ BatchBlock batch_block() {
    const unsigned nb = gridDim.y, gx = gridDim.x;
    const unsigned w = blockIdx.y * gx + blockIdx.x;
    const unsigned xcd = w & 7u, r = w >> 3;
    BatchBlock bb;
    if ((nb & 7u) == 0) {
        const unsigned k = nb >> 3;
        bb.j = (int)(xcd + 8u * (r % k));
        bb.x = r / k;
    } else if (nb < 8 && (8u % nb) == 0 && (gx & 7u) == 0) {
        const unsigned k = 8u / nb;
        bb.j = (int)(xcd % nb);
        bb.x = r * k + xcd / nb;
    } else {
        bb.j = (int)blockIdx.y;
        bb.x = blockIdx.x;
    }
    return bb;
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

// The same scan for several independent sequences at once, in two launches; batch_block() names the
// sequence ("batch") j.
//   In:  int64_t n(int j) const (length, read on the device; the second launch calls n(j, total) with the
//        sequence's total); int operator()(int j, int64_t i) const
//   Out: void operator()(int j, int64_t i, int ex, int v, int total) const
//   Fin: void operator()(int j, int total) const      called once per sequence, by one thread
// `partial` holds gridDim.x ints per sequence.  Every workgroup of the second launch adds up the
// partial sums of its sequence itself (there are a few dozen), so no launch stands between the two
// passes; Fin runs at the start of the second launch, in workgroup 0 of the sequence, which means
// that the other workgroups of that launch must not depend on what Fin writes: n(j, total), Out
// and Tail get the sequence's total and derive what they need from it.  (Where Fin sets a flag
// that those workgroups also read, they combine it with the launch-invariant condition under
// which Fin sets it, so that either value of the flag gives the same outcome.)
// Two hooks let independent work ride in the same launches (a launch costs more than most of
// these steps): Head: void operator()(int j, unsigned x, unsigned gx) const runs before the
// reduction, Tail: void operator()(int j, unsigned x, unsigned gx, int total) const after the write
// pass; x is the workgroup's index among the gx of sequence j.
struct NoHook {
    __device__ void operator()(int, unsigned, unsigned) const {}
    __device__ void operator()(int, unsigned, unsigned, int) const {}
};

template <class In, class Head>
__global__ void __launch_bounds__(kBlock) bscan_reduce_kernel(In in, int* partial, Head head) {
    __shared__ int lds[4];
    const BatchBlock bb = batch_block();
    const int j = bb.j;
    head(j, bb.x, gridDim.x);
    int64_t b, e;
    scan_range(in.n(j), bb.x, b, e);
    int acc = 0;
    for (int64_t i = b + threadIdx.x; i < e; i += kBlock) acc = uadd(acc, in(j, i));
    int t = block_reduce_sum(acc, lds);
    if (threadIdx.x == 0) partial[(int64_t)j * gridDim.x + bb.x] = t;
}

template <class In, class Out, class Fin, class Tail>
__global__ void __launch_bounds__(kBlock) bscan_write_kernel(In in, Out out, Fin fin, const int* partial, Tail tail) {
    __shared__ int lds[4];
    const BatchBlock bb = batch_block();
    const int j = bb.j;
    // this workgroup's prefix and the sequence's total, from the partial sums of the first launch
    const int* p = partial + (int64_t)j * gridDim.x;
    int carry = 0, seq_total = 0;
    for (unsigned base = 0; base < gridDim.x; base += kBlock) {
        const unsigned i = base + threadIdx.x;
        const int v = i < gridDim.x ? p[i] : 0;
        seq_total = uadd(seq_total, block_reduce_sum(v, lds));
        carry = uadd(carry, block_reduce_sum(i < bb.x ? v : 0, lds));
    }
    if (bb.x == 0 && threadIdx.x == 0) fin(j, seq_total);
    int64_t b, e;
    scan_range(in.n(j, seq_total), bb.x, b, e);
    for (int64_t base = b; base < e; base += kBlock) {
        int64_t i = base + threadIdx.x;
        int v = i < e ? in(j, i) : 0;
        int total;
        int ex = block_exclusive_scan(v, lds, total);
        if (i < e) out(j, i, uadd(carry, ex), v, seq_total);
        carry = uadd(carry, total);
    }
    tail(j, bb.x, gridDim.x, seq_total);
}

template <class In, class Out, class Fin, class Head = NoHook, class Tail = NoHook>
inline void grid_scan_batched(hipStream_t st, int grid, int nbatch, In in, Out out, Fin fin, int* partial,
                              Head head = Head(), Tail tail = Tail()) {
    bscan_reduce_kernel<In, Head><<<dim3(grid, nbatch), kBlock, 0, st>>>(in, partial, head);
    bscan_write_kernel<In, Out, Fin, Tail><<<dim3(grid, nbatch), kBlock, 0, st>>>(in, out, fin, partial, tail);
}

// The same with a value function of its own for the second launch (one that reads what the first
// launch's function left behind instead of computing the value again).
template <class In, class In2, class Out, class Fin, class Head = NoHook, class Tail = NoHook>
inline void grid_scan_batched_two(hipStream_t st, int grid, int nbatch, In in, In2 in2, Out out, Fin fin, int* partial,
                                  Head head = Head(), Tail tail = Tail()) {
    bscan_reduce_kernel<In, Head><<<dim3(grid, nbatch), kBlock, 0, st>>>(in, partial, head);
    bscan_write_kernel<In2, Out, Fin, Tail><<<dim3(grid, nbatch), kBlock, 0, st>>>(in2, out, fin, partial, tail);
}

// ---------------------------------------------------------------------------------------------
// Open-addressing table of 64-bit entries (key << 32 | value), empty = all ones.  Keys are vertex
// ids (below 2^31).  The capacity is a power of two >= 1024 and at least twice the number of keys.
// A key hashes to a slot; a probe reads the slot's whole bucket of 8 (one 64-byte line) with four
// 128-bit loads and walks it from the hashed slot round to the slot before it, then does the same
// in the next bucket with the same starting offset: at half load nearly every lookup ends in the
// first bucket, so a lookup costs one memory round trip (the kernels that use the table are bound
// by that latency, not by bandwidth), and keys of one bucket start at different slots, so
// concurrent insertions seldom compete for the same empty slot.
// The bucket is read with plain loads, which may return an older state of a slot.  That is safe:
// a slot's key is written once (by the compare-and-swap that claims it) and its value only ever
// decreases, so an old view can only show a claimed slot as still empty, where the
// compare-and-swap then fails and returns the current entry, or show a larger value, where the
// atomic minimum still applies.  Lookups run in later launches than the insertions they read.
// ---------------------------------------------------------------------------------------------
constexpr uint64_t kEmpty = ~0ull;
constexpr int kBucketSlots = 8;

__device__ __forceinline__ uint32_t table_hash(uint32_t key, int shift) {
    return (key * 0x9E3779B1u) >> shift;         // top log2(capacity) bits of a Fibonacci product
}

// s[idx] for a run-time idx without indexing registers through memory
__device__ __forceinline__ unsigned long long table_pick(const unsigned long long (&s)[8], uint32_t idx) {
    const unsigned long long a = (idx & 1u) ? s[1] : s[0];
    const unsigned long long b = (idx & 1u) ? s[3] : s[2];
    const unsigned long long c = (idx & 1u) ? s[5] : s[4];
    const unsigned long long d = (idx & 1u) ? s[7] : s[6];
    const unsigned long long ab = (idx & 2u) ? b : a;
    const unsigned long long cd = (idx & 2u) ? d : c;
    return (idx & 4u) ? cd : ab;
}

__device__ __forceinline__ void table_load_bucket(const unsigned long long* tab, uint32_t b,
                                                  unsigned long long (&s)[kBucketSlots]) {
    typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));
    const u64x2* p = reinterpret_cast<const u64x2*>(tab + (size_t)b * kBucketSlots);
#pragma unroll
    for (int k = 0; k < kBucketSlots / 2; ++k) {
        const u64x2 v = p[k];
        s[2 * k] = v.x;
        s[2 * k + 1] = v.y;
    }
}

// Keeps, per key, the smallest value ever offered; returns the slot that holds the key.
// `mask` = capacity - 1, `shift` = 32 - log2(capacity).
__device__ __forceinline__ uint32_t table_insert_min(unsigned long long* tab, uint32_t mask, int shift,
                                                     uint32_t key, uint32_t value) {
    const unsigned long long want = ((unsigned long long)key << 32) | value;
    const uint32_t bmask = mask >> 3;
    const uint32_t h0 = table_hash(key, shift);
    uint32_t b = h0 >> 3;
    for (;;) {
        unsigned long long s[kBucketSlots];
        table_load_bucket(tab, b, s);
#pragma unroll
        for (int k = 0; k < kBucketSlots; ++k) {
            const uint32_t idx = (h0 + k) & 7u;
            unsigned long long cur = table_pick(s, idx);
            const uint32_t h = b * kBucketSlots + idx;
            if ((uint32_t)(cur >> 32) == 0xFFFFFFFFu) {          // seen empty: claim it
                const unsigned long long old = atomicCAS(&tab[h], (unsigned long long)kEmpty, want);
                if (old == kEmpty) return h;
                cur = old;                                       // someone else's entry, current
            }
            if ((uint32_t)(cur >> 32) == key) {
                if (want < cur) atomicMin(&tab[h], want);
                return h;
            }
        }
        b = (b + 1) & bmask;
    }
}

// Claims `key` for `value` if no entry holds the key yet.  Returns true to the one thread that
// placed the entry; every other thread asking for the same key gets false and the claimer's value
// in `existing` (an entry is never changed once placed, so a stale view is harmless as above).
__device__ __forceinline__ bool table_claim(unsigned long long* tab, uint32_t mask, int shift, uint32_t key,
                                            uint32_t value, uint32_t& existing) {
    const unsigned long long want = ((unsigned long long)key << 32) | value;
    const uint32_t bmask = mask >> 3;
    const uint32_t h0 = table_hash(key, shift);
    uint32_t b = h0 >> 3;
    for (;;) {
        unsigned long long s[kBucketSlots];
        table_load_bucket(tab, b, s);
#pragma unroll
        for (int k = 0; k < kBucketSlots; ++k) {
            const uint32_t idx = (h0 + k) & 7u;
            unsigned long long cur = table_pick(s, idx);
            if ((uint32_t)(cur >> 32) == 0xFFFFFFFFu) {
                const unsigned long long old = atomicCAS(&tab[b * kBucketSlots + idx], (unsigned long long)kEmpty, want);
                if (old == kEmpty) return true;
                cur = old;
            }
            if ((uint32_t)(cur >> 32) == key) { existing = (uint32_t)cur; return false; }
        }
        b = (b + 1) & bmask;
    }
}

// Returns the slot index of `key`, or -1; `value` receives the stored value.
__device__ __forceinline__ int64_t table_find(const unsigned long long* tab, uint32_t mask, int shift,
                                              uint32_t key, uint32_t& value) {
    const uint32_t bmask = mask >> 3;
    const uint32_t h0 = table_hash(key, shift);
    uint32_t b = h0 >> 3;
    for (;;) {
        unsigned long long s[kBucketSlots];
        table_load_bucket(tab, b, s);
#pragma unroll
        for (int k = 0; k < kBucketSlots; ++k) {
            const uint32_t idx = (h0 + k) & 7u;
            const unsigned long long cur = table_pick(s, idx);
            if (cur == kEmpty) return -1;
            if ((uint32_t)(cur >> 32) == key) { value = (uint32_t)cur; return (int64_t)b * kBucketSlots + idx; }
        }
        b = (b + 1) & bmask;
    }
}

// ---------------------------------------------------------------------------------------------
// Edges grouped by blocks of destination rows and sorted by source inside a block, one 32-bit word
// per edge: (source & (2^18 - 1)) << 14 | row inside the block.  The source's high bits are the
// index of its "source chunk"; bound[c] is the position inside the block of the first edge whose
// chunk is >= c (bound[0] = 0, bound[nch] = edges of the block), so the chunk of the edge at
// position p is the largest c with bound[c] <= p.
// ---------------------------------------------------------------------------------------------
constexpr int kTileSrcLoBits = 18;
constexpr int kTileRowBits = 14;
constexpr uint32_t kTileRowMask = (1u << kTileRowBits) - 1u;

__device__ __forceinline__ int tile_chunk_of(const uint32_t* bound, int nch, uint32_t p) {
    int lo = 0, hi = nch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (bound[mid] <= p) lo = mid; else hi = mid - 1;
    }
    return lo;
}
__device__ __forceinline__ uint32_t tile_source(uint32_t word, int chunk) {
    return ((uint32_t)chunk << kTileSrcLoBits) | (word >> kTileRowBits);
}

// The chunked layout of the same edges: chunks of 2^kXSrcBits sources, row blocks of 2^kTileRowBits
// rows; an entry is a 16-bit source inside its chunk (kXPad marks padding) and a 16-bit row inside
// its block.
constexpr int kXSrcBits = 15;
constexpr uint32_t kXPad = 0x8000u;
constexpr int kXGroup = 2048;            // pieces of a row block whose table entries sit in LDS at a time
constexpr int64_t kChunkedAboveVertices = (int64_t)1 << 23;   // graphs with more vertices get the chunked layout

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
