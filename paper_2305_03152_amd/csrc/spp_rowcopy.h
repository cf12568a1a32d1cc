// Row-copy kernels shared by the gather and the cache fill.  A row of `row_bytes` bytes is cut
// into vectors of V bytes (V = 16 when sizes and addresses allow: one 128-bit load and store per
// lane); the output is walked as one flat array of vectors, so stores are fully coalesced and
// every lane is busy whatever the row size, while loads are coalesced within a row.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spp_common.h"
#include "spp_device.h"

namespace spp {

template <int V> struct VecOf;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <> struct VecOf<16> { typedef u32x4 type; };
template <> struct VecOf<8>  { typedef u32x2 type; };
template <> struct VecOf<4>  { typedef uint32_t type; };
template <> struct VecOf<2>  { typedef uint16_t type; };

// Source descriptor of an output row: tag in the top three bits, row index in the store below.
// kTagLocal: row of the device-resident local rows; kTagLocalHost: row of the host-resident ones;
// kTagDup: the same remote vertex is fetched for another output row of this call, whose virtual
// row is stored: this row is copied from that one once it has arrived.
constexpr int kTagLocal = 0, kTagCache = 1, kTagMiss = 2, kTagSkip = 3, kTagLocalHost = 4, kTagDup = 5;
__device__ __host__ __forceinline__ int64_t make_desc(int tag, int64_t row) { return (int64_t)((uint64_t)tag << 61) | row; }
__device__ __forceinline__ int desc_tag(int64_t d) { return (int)(((uint64_t)d) >> 61); }
__device__ __forceinline__ int64_t desc_row(int64_t d) { return d & ((1ll << 61) - 1); }

template <int V>
__device__ __forceinline__ typename VecOf<V>::type load_stream(const void* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const typename VecOf<V>::type*>(p));
}
template <int V>
__device__ __forceinline__ void store_stream(void* p, typename VecOf<V>::type v) {
    __builtin_nontemporal_store(v, reinterpret_cast<typename VecOf<V>::type*>(p));
}

constexpr int kCopyUnroll = 4;          // vectors in flight per lane, indexed (PCIe) copy
constexpr int kHitUnroll = 4;           // vectors in flight per lane, hit copy
constexpr int64_t kListAlign = 2048;    // every list starts at a multiple of this in the virtual row space

// The offsets and counts are read many times by every workgroup: a copy in LDS keeps the search for
// a row's list off the global-memory latency path.
struct ListLds {
    int64_t off[kMaxLists + 1];
    int64_t cnt[kMaxLists];
    char*   out[kMaxLists];     // a lane picks its list at run time: from LDS, not from the argument block
};
__device__ __forceinline__ void load_lists(const ListTable& t, ListLds& s) {
    if (threadIdx.x <= (unsigned)t.n_lists) s.off[threadIdx.x] = t.off[threadIdx.x];
    if (threadIdx.x < (unsigned)t.n_lists) { s.cnt[threadIdx.x] = t.cnt[threadIdx.x]; s.out[threadIdx.x] = t.out[threadIdx.x]; }
    __syncthreads();
}
// Index of the list that owns virtual row r (r < off[n_lists]).
__device__ __forceinline__ int list_of(const ListLds& s, int n_lists, int64_t r) {
    int lo = 0, hi = n_lists - 1;                 // last j with off[j] <= r
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (r >= s.off[mid]) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Hit path: rows served from the local shard or the cache.  The classification leaves, for every
// chunk of kListAlign consecutive virtual rows, the chunk's hits in row order in the chunk's own
// part of the hit list (hitlist[chunk * kListAlign + i], i < hcount[chunk]), so the list needs no
// global cursor and the copy walks the outputs in order (with chunks appended to one list in the
// order in which workgroups finished, the same copy was 5 to 9 % slower).
// A hit-list entry names the output row and its source in one 64-bit word (bit 63: cache instead
// of local shard, bits 32-62: row in that store, bits 26-31: list, bits 0-25: row in the list's
// output), so a lane reaches the source row with one dependent load.  Only hits are walked, so
// every lane copies (no lane idles on a row that missed).
// Source rows are read with ordinary loads (hot rows of the shard and the cache stay in L2 and
// the Infinity Cache across batches), the output is written with streaming stores (it is not read
// again by this path).
constexpr int kHitRowBits = 26;         // rows of one list that a hit-list entry can name
static_assert(SPP_MAX_GATHER_LISTS <= (1 << (32 - kHitRowBits)), "the list index has 32 - kHitRowBits bits");
__device__ __forceinline__ int64_t make_hit(bool from_cache, int64_t src_row, int list, int64_t row_in_list) {
    return (int64_t)(((uint64_t)(from_cache ? 1 : 0) << 63) | ((uint64_t)src_row << 32) |
                     ((uint64_t)list << kHitRowBits) | (uint64_t)row_in_list);
}
// A work item is one tile of kBlock * U consecutive vectors of one chunk's hits (every lane U
// vectors, all loads issued before the first store), so items are equal whatever the chunk holds,
// except the last tile of a chunk; a chunk has tiles_per_chunk of them (enough for 2048 hits), and
// tiles beyond the chunk's hits are skipped.  (Cutting every chunk into 16 slices of hits/16 rows
// instead left the last round of most slices two thirds full: 5.2 TB/s on 256-byte rows of a
// 3.5 GB shard where tiles reach 5.5 on the same box.  One, two, four or eight vectors per lane:
// four is best by 1 to 4 %; non-temporal loads of the source rows cost 4 % when the shard is in
// HBM and 25 % when it fits the Infinity Cache.)
// The tiles that hold hits, listed: item_list[i] = chunk << 32 | tile << 16 | the tile's vectors,
// i < *n_items, in the order of the chunks (an entry says all a workgroup needs to start loading).  Without the list a copy's workgroups take every tile a chunk could
// have and leave at once where the chunk's hits end; a list that misses a tenth of its ids then
// strews a tenth of empty workgroups among the busy ones, each of which waits out a load behind
// the copy's own traffic before it can leave (5 % of the copy's time on 256-byte rows).  With the
// list the surplus workgroups are the last of the grid.  One workgroup per id list: it adds up the
// tiles of the lists before it (a few thousand chunk counts at most) and then numbers its own.
constexpr int kHitTileBits = 16;         // tiles of a chunk that an entry of the list can name
template <int V, int U = kHitUnroll>
__global__ void __launch_bounds__(kBlock) gather_hit_kernel(const int64_t* __restrict__ hitlist,
                                                            const int32_t* __restrict__ hcount, ListTable t,
                                                            const char* __restrict__ local,
                                                            const char* __restrict__ cache, uint32_t vpr,
                                                            uint32_t tiles_per_chunk, const uint64_t* __restrict__ item_list,
                                                            const uint32_t* __restrict__ n_items, int64_t item_cap) {
    typedef typename VecOf<V>::type vec_t;
    // one tile: vectors [base, nv) of the chunk's hits, kBlock * U of them at most
    auto copy_tile = [&](int64_t chunk, uint32_t base, uint32_t nv) {
        const int64_t* __restrict__ hl = hitlist + chunk * kListAlign;
        vec_t v[U];
        char* dst[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = base + (uint32_t)u * kBlock + threadIdx.x;
            ok[u] = c < nv;
            if (ok[u]) {
                const uint32_t m = c / vpr;
                const uint32_t k = c - m * vpr;
                const uint64_t h = (uint64_t)hl[m];
                const uint64_t srow = (h >> 32) & 0x7FFFFFFFull;
                const char* src = ((h >> 63) ? cache : local) + (srow * vpr + k) * (uint64_t)V;
                v[u] = *reinterpret_cast<const vec_t*>(src);
                const uint32_t lo = (uint32_t)h;
                // a chunk belongs to one list: its output pointer is the same for all lanes
                char* out = t.out[__builtin_amdgcn_readfirstlane((int)(lo >> kHitRowBits))];
                dst[u] = out + ((uint64_t)(lo & ((1u << kHitRowBits) - 1u)) * vpr + k) * (uint64_t)V;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ok[u]) store_stream<V>(dst[u], v[u]);
    };
    if (item_list) {
        // the list of the tiles that hold hits: the workgroup's first entry is asked for together with the
        // list's length (entries beyond the length are stale and never used), so a workgroup's rows are two
        // round trips away from its start
        int64_t w = blockIdx.x;
        uint64_t e = w < item_cap ? item_list[w] : 0ull;
        const int64_t items = (int64_t)*n_items;
        while (w < items) {
            const uint32_t base = ((uint32_t)e >> kHitTileBits) * (uint32_t)(kBlock * U);
            copy_tile((int64_t)(e >> 32), base, base + ((uint32_t)e & ((1u << kHitTileBits) - 1u)));
            w += gridDim.x;
            if (w < items) e = item_list[w];
        }
        return;
    }
    // without the list: every tile of every chunk in use
    const int64_t items = t.off[t.n_lists] / kListAlign * tiles_per_chunk;
    for (int64_t w = blockIdx.x; w < items; w += gridDim.x) {
        const int64_t chunk = w / tiles_per_chunk;
        const uint32_t base = (uint32_t)(w - chunk * tiles_per_chunk) * (uint32_t)(kBlock * U);
        const uint32_t nv = (uint32_t)hcount[chunk] * vpr;                 // at most 2048 rows: fits 32 bits
        if (base < nv) copy_tile(chunk, base, nv);
    }
}

// Miss path: rows read straight from the remote store (pinned host memory over PCIe, or device
// memory), or from the host-resident part of the local rows.  misslist[m] is a virtual row; its
// descriptor names the store and the row in it.
template <int V, int BS = kBlock>
__global__ void __launch_bounds__(BS) gather_miss_kernel(const char* __restrict__ src,
                                                             const char* __restrict__ local_host,
                                                             const int64_t* __restrict__ desc,
                                                             const int32_t* __restrict__ misslist,
                                                             const int64_t* __restrict__ count_ptr, ListTable t,
                                                             uint32_t vpr) {
    typedef typename VecOf<V>::type vec_t;
    __shared__ ListLds ls;
    load_lists(t, ls);
    const uint64_t total = (uint64_t)(*count_ptr) * vpr;
    const bool small = total <= 0xFFFFFFFFull;
    const uint64_t span = (uint64_t)BS * kCopyUnroll;
    for (uint64_t base = (uint64_t)blockIdx.x * span; base < total; base += (uint64_t)gridDim.x * span) {
        vec_t v[kCopyUnroll];
        char* dst[kCopyUnroll];
        bool ok[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const uint64_t c = base + (uint64_t)u * BS + threadIdx.x;
            ok[u] = c < total;
            if (ok[u]) {
                const uint64_t m = small ? (uint64_t)((uint32_t)c / vpr) : c / vpr;
                const uint32_t k = (uint32_t)(c - m * vpr);
                const int64_t r = misslist[m];
                const int64_t d = r >= 0 ? desc[r] : 0;
                const int j = r >= 0 ? list_of(ls, t.n_lists, r) : 0;
                const char* from = desc_tag(d) == kTagLocalHost ? local_host : src;
                // struck from the list (another row fetches the vertex), or a store the caller did
                // not give: the row is left to the copy pass, or untouched (the statistics report it)
                ok[u] = r >= 0 && from != nullptr;
                if (ok[u]) {
                    v[u] = load_stream<V>(from + ((uint64_t)desc_row(d) * vpr + k) * (uint64_t)V);
                    dst[u] = ls.out[j] + ((uint64_t)(r - ls.off[j]) * vpr + k) * (uint64_t)V;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (ok[u]) store_stream<V>(dst[u], v[u]);
    }
}

// Rows whose vertex another row of the same call fetches from the host: copied from that row's
// output (device memory) after the miss copy, so a vertex that several minibatches of the call
// miss crosses PCIe once.
template <int V>
__global__ void __launch_bounds__(kBlock) gather_dup_kernel(const int64_t* __restrict__ desc,
                                                            const int32_t* __restrict__ duplist,
                                                            const int64_t* __restrict__ count_ptr, ListTable t,
                                                            uint32_t vpr) {
    typedef typename VecOf<V>::type vec_t;
    __shared__ ListLds ls;
    load_lists(t, ls);
    const uint64_t total = (uint64_t)(*count_ptr) * vpr;
    for (uint64_t c = (uint64_t)blockIdx.x * kBlock + threadIdx.x; c < total; c += (uint64_t)gridDim.x * kBlock) {
        const uint64_t m = c / vpr;
        const uint32_t k = (uint32_t)(c - m * vpr);
        const int64_t r = duplist[m];
        const int64_t rs = desc_row(desc[r]);
        const int j = list_of(ls, t.n_lists, r), js = list_of(ls, t.n_lists, rs);
        const vec_t v = *reinterpret_cast<const vec_t*>(ls.out[js] + ((uint64_t)(rs - ls.off[js]) * vpr + k) * (uint64_t)V);
        store_stream<V>(ls.out[j] + ((uint64_t)(r - ls.off[j]) * vpr + k) * (uint64_t)V, v);
    }
}

// Cache fill: out[m,:] = src[rowidx[m],:], m < count, from a store that may be pinned host memory.
template <int V>
__global__ void __launch_bounds__(kBlock) rows_indexed_kernel(const char* __restrict__ src,
                                                              const int64_t* __restrict__ rowidx, int64_t count,
                                                              uint32_t vpr, char* __restrict__ out) {
    typedef typename VecOf<V>::type vec_t;
    const uint64_t total = (uint64_t)count * vpr;
    const bool small = total <= 0xFFFFFFFFull;
    const uint64_t span = (uint64_t)kBlock * kCopyUnroll;
    for (uint64_t base = (uint64_t)blockIdx.x * span; base < total; base += (uint64_t)gridDim.x * span) {
        vec_t v[kCopyUnroll];
        bool ok[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const uint64_t c = base + (uint64_t)u * kBlock + threadIdx.x;
            ok[u] = c < total;
            if (ok[u]) {
                const uint64_t m = small ? (uint64_t)((uint32_t)c / vpr) : c / vpr;
                const uint32_t k = (uint32_t)(c - m * vpr);
                v[u] = load_stream<V>(src + ((uint64_t)rowidx[m] * vpr + k) * (uint64_t)V);
            }
        }
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) {
            const uint64_t c = base + (uint64_t)u * kBlock + threadIdx.x;
            if (ok[u]) store_stream<V>(out + c * (uint64_t)V, v[u]);
        }
    }
}

// Widest vector that divides the row size and is honoured by every address.
inline int pick_vec(int64_t row_bytes, uintptr_t address_bits) {
    const uintptr_t bits = (uintptr_t)row_bytes | address_bits;
    if ((bits & 15) == 0) return 16;
    if ((bits & 7) == 0) return 8;
    if ((bits & 3) == 0) return 4;
    return 2;
}

}  // namespace spp
