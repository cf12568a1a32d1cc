// Shared host-side plumbing of the library: error reporting, handle layouts, workspace helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include <string.h>
#include <stdlib.h>

#include <vector>

#include "../../include/spp.h"

namespace spp {

void set_error(const char* fmt, ...);

#define SPP_HIP(call)                                                                       \
    do {                                                                                    \
        hipError_t e__ = (call);                                                            \
        if (e__ != hipSuccess) {                                                            \
            spp::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e__), __FILE__, \
                           __LINE__);                                                       \
            return (e__ == hipErrorOutOfMemory) ? SPP_E_OOM : SPP_E_HIP;                    \
        }                                                                                   \
    } while (0)

#define SPP_CHECK(cond, code, ...)                                                          \
    do {                                                                                    \
        if (!(cond)) {                                                                      \
            spp::set_error(__VA_ARGS__);                                                    \
            return (code);                                                                  \
        }                                                                                   \
    } while (0)

#define SPP_TRY(expr)                                                                       \
    do {                                                                                    \
        int rc__ = (expr);                                                                  \
        if (rc__ != SPP_OK) return rc__;                                                    \
    } while (0)

// A grow-only device buffer owned by a context.
struct DevBuf {
    void*  ptr = nullptr;
    size_t bytes = 0;
    int reserve(size_t need) {
        if (need <= bytes) return SPP_OK;
        if (ptr) { (void)hipFree(ptr); ptr = nullptr; bytes = 0; }
        size_t want = need + need / 8 + 256;
        hipError_t e = hipMalloc(&ptr, want);
        if (e != hipSuccess) {
            ptr = nullptr;
            set_error("hipMalloc of %zu bytes failed: %s", want, hipGetErrorString(e));
            return SPP_E_OOM;
        }
        bytes = want;
        return SPP_OK;
    }
    void release() { if (ptr) (void)hipFree(ptr); ptr = nullptr; bytes = 0; }
    template <class T> T* as() const { return reinterpret_cast<T*>(ptr); }
};

constexpr int kNumTimers = SPP_T_COUNT;

// Several id lists gathered by one set of launches.  List j owns the virtual rows
// [off[j], off[j] + cnt[j]); off[] is padded to multiples of kListAlign so that one workgroup's
// chunk of rows (or of vectors) never straddles two lists.
constexpr int kMaxLists = SPP_MAX_GATHER_LISTS;
struct ListTable {
    const int32_t* ids[kMaxLists];
    char*          out[kMaxLists];
    const int64_t* off;     // device int64[n_lists + 1]
    const int64_t* cnt;     // device int64[n_lists]
    int            n_lists;
};

// What is left to do for a gather whose miss copy was left running on the side stream: wait for
// it, then copy the rows that share a fetched vertex from the rows that fetched them.
struct PendingGather {
    bool           active = false;
    int            slot = 0;            // which join event the miss copy records
    bool           has_dup = false;
    int            V = 0;               // vector width of the copy
    uint32_t       vpr = 0;
    const int64_t* desc = nullptr;
    const int32_t* duplist = nullptr;
    const int64_t* dup_count = nullptr;
    ListTable      t;
};

}  // namespace spp

struct spp_ctx {
    int         device = 0;
    hipStream_t stream = nullptr;       // caller's stream
    hipStream_t side = nullptr;         // miss path
    hipEvent_t  ev_fork = nullptr, ev_join[2] = {nullptr, nullptr};   // one join event per workspace set
    spp::PendingGather pending;         // the gather whose miss copy is still running on the side stream
    int         num_cu = 256;
    // sampling workspaces
    spp::DevBuf table;                  // uint64 hash table: global id -> local id / first position
    spp::DevBuf flat;                   // int32 sampled global ids of the current hop
    spp::DevBuf nodeinfo;               // per minibatch: row start and length of the vertices of S_{L-1}
    spp::DevBuf slots;                  // per minibatch: mask and shift of the id table of the current hop
    spp::DevBuf partials;               // scan partial sums
    // sampler: the per-call table of per-minibatch pointers is kept on the device in a few slots and stored again
    // only when a call brings other buffers (a pipeline alternates between a few buffer sets); two sets of error
    // flags, used alternately, the next call's cleared by the last kernel of this one
    static constexpr int kBatchSlots = 4;
    spp::DevBuf btab;                   // kBatchSlots tables, then the flags
    void*       btab_mirror = nullptr;  // host copies of what the slots hold (malloc)
    int         btab_n[kBatchSlots] = {};        // minibatches in each slot's table (0: empty)
    uint64_t    btab_stamp[kBatchSlots] = {};    // last use
    uint64_t    sample_calls = 0;
    int         sample_flags_clean = 0; // the flags of the next call have been cleared on the stream
    // gather workspaces
    // two sets, used alternately: the classification of a call may run while the miss copy of the
    // call before still reads its own set
    spp::DevBuf srcdesc[2];             // int64 per row: where the row comes from
    spp::DevBuf misslist[2];            // the lists of a call: rows that hit (64-bit entries), miss, share a fetch, miss in store order
    spp::DevBuf gcount[2];              // device counters of the gather (int64[8]) and the list layout
    spp::DevBuf hititems[2];            // the hit copy's work items (chunk, tile) that hold hits, and their number
    int         gslot = 0;              // set used by the last gather
    int         miss_lds = 0;           // dynamic LDS bytes of the miss kernel
    spp::DevBuf gtable;                 // vertices missed by the current gather call (id -> first row)
    spp::DevBuf gfirst;                 // the same per row of the remote store (SPP_STORE_ORDER): first row that misses it
    int64_t*    h_pinned = nullptr;     // pinned host mirror (8192 int64): gather counters from 40, sampler counts from 64,
                                        // per-workgroup frontier sizes of the VIP propagation from 2048
    int64_t*    totals = nullptr;       // device int64[16], running sums since the last reset (see spp_ctx_totals)
    // vip workspaces
    spp::DevBuf y0, y1, tot, acc, frontier;
    spp::DevBuf xvals;                  // dense hops over the chunked layout: y[source] of every entry
    spp::DevBuf bins;                   // general propagation: per row block the (row, weight) entries of a hop, and the fill counts
    int         bin_lds_set = 0, sum_lds_set = 0;   // dynamic LDS bytes its two kernels have been allowed
    int         tile_lds_set = 0;       // dynamic LDS bytes the dense-hop kernel has been allowed on this device
    int         dedup_lds_set = 0;      // the LDS dedup kernel of the sampler has been allowed its 128 KB
    int         x_lds_set = 0;          // the two kernels of the chunked layout have been allowed theirs
    int         vip_pushed[SPP_MAX_L] = {};          // last vip_propagate: hop done in push form?
    int64_t     vip_frontier_edges[SPP_MAX_L] = {};  // last vip_propagate: out-edges of each hop's frontier
    // timing: while enabled every timed piece of device work gets its own pair of events
    int         timing = 0;
    struct Span { int idx; hipEvent_t t0, t1; };
    std::vector<hipEvent_t> ev_free;
    std::vector<Span>       spans;
    hipEvent_t take_event() {
        if (!ev_free.empty()) { hipEvent_t e = ev_free.back(); ev_free.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};

struct spp_graph {
    int            device = 0;          // handles outlive contexts: they keep the device, not the context
    int64_t        N = 0, M = 0;
    const int64_t* rowptr = nullptr;    // caller's
    const int32_t* col = nullptr;       // caller's
    // the same edges once more (library-owned, built on request), grouped by blocks of
    // 2^tile_rbits destination rows and sorted by source inside a block: the structure the
    // dense hops of the VIP propagation walk.  One 32-bit word per edge: the low kTileSrcLoBits of
    // the source above the destination row inside its block; the high bits of the source are the
    // index of the "source chunk", and tile_first says where each chunk starts inside each block.
    bool      has_in = false;
    uint32_t* t_edge = nullptr;         // uint32[M]
    int64_t*  tile_first = nullptr;     // int64[nrb * nch + 1]: first edge of (row block, source chunk), ascending
    int       tile_rbits = 0;
    int64_t   nrb = 0;                  // row blocks
    int       nch = 0;                  // source chunks (of 2^kTileSrcLoBits vertices)
    int64_t*  block_first = nullptr;    // int64[nrb + 1]: edges that end in row blocks before b (either layout)
    // The second layout of the same edges, built instead of the first for graphs whose per-vertex
    // vector is too large to be gathered from (see spp_vip.hip): the edges sorted by (chunk of 2^15
    // sources, row block, source), every (chunk, row block) piece padded to a multiple of four
    // entries, 2 + 2 bytes per entry.  A dense hop first writes y[source] for every entry in this
    // order (a chunk of y sits in LDS), then every row block adds up its pieces.
    bool      has_x = false;
    uint16_t* x_src = nullptr;          // uint16[x_entries]: source inside its chunk; bit 15: padding
    uint16_t* x_row = nullptr;          // uint16[x_entries]: row inside its block
    int64_t*  x_chunk_first = nullptr;  // int64[x_nch + 1]: first entry of chunk c
    uint32_t* x_start = nullptr;        // uint32[nrb * x_nch]: piece (b, c): its first vector (four entries) in the arrays
    uint32_t* x_prefix = nullptr;       // uint32[nrb * (x_nch + 1)]: vectors of row block b in chunks before c
    int64_t   x_entries = 0;
    int       x_nch = 0;
};

struct spp_cache {
    int       device = 0;
    int64_t   N = 0, lo = 0, hi = 0;
    int64_t   n_rows = 0;               // rows built
    int64_t   limit = 0;                // rows in use (<= n_rows)
    int64_t   row_bytes = 0;
    uint64_t* table = nullptr;          // (id << 32 | slot), empty = ~0
    uint32_t  table_mask = 0;
    int       table_shift = 0;
    void*     rows = nullptr;           // [n_rows, row_bytes] or null (membership only)
};

struct spp_local_store {
    int       device = 0;
    int64_t   N = 0, lo = 0, hi = 0;
    int64_t   n_rows = 0;               // rows held in device memory
    int64_t   limit = 0;                // rows in use (<= n_rows)
    int64_t   row_bytes = 0;
    int32_t*  rank = nullptr;           // [hi-lo] position of every local vertex in the order
    void*     rows = nullptr;           // [n_rows, row_bytes], in rank order
    const void* host_rows = nullptr;    // the caller's [hi-lo, row_bytes] (device-visible address)
};

namespace spp {


struct ScopedTimer {
    spp_ctx* c; int idx; hipStream_t s; hipEvent_t a = nullptr, b = nullptr;
    ScopedTimer(spp_ctx* ctx, int i, hipStream_t st) : c(ctx), idx(i), s(st) {
        if (!c->timing) return;
        a = c->take_event(); b = c->take_event();
        if (a && b) (void)hipEventRecord(a, s);
    }
    ~ScopedTimer() {
        if (!c->timing || !a || !b) return;
        (void)hipEventRecord(b, s);
        c->spans.push_back({idx, a, b});
    }
};

// 64-bit LSD radix sort of `n` keys on bits [bit_lo, bit_hi); stable.  keys_a holds the input and,
// on return, *result points at whichever of keys_a / keys_b holds the sorted output.
int radix_sort_u64(spp_ctx* ctx, uint64_t* keys_a, uint64_t* keys_b, int64_t n, int bit_lo,
                   int bit_hi, uint64_t** result);

// Device-visible address of a row store that is either device memory or pinned host memory.
int device_view(const void* p, const void** out);
// Address, on the current device `device`, of the fixed workspace of spp_gather_features_static
// (looked up once per device).
int static_scratch(int device, void** out);
// Rows copied from a row store that may be pinned host memory: out[i,:] = src[rows[i],:].
int copy_rows_indexed(hipStream_t st, const void* src, const int64_t* d_rowidx, int64_t n,
                      int64_t row_bytes, void* d_out, int num_cu);

// Slots of an id table for x/2 keys: the smallest power of two >= x, at most 2^31 (a table index
// has 32 bits; key counts stay below 2^31, so such a table still has a free slot).
static inline uint32_t next_pow2(uint64_t x) {
    uint64_t p = 1;
    while (p < x && p < (1ull << 31)) p <<= 1;
    return (uint32_t)p;
}

}  // namespace spp
