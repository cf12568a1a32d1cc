// Cache-aware feature gather (Secs. 4.1-4.3; stages 5-10 of the pipeline walkthrough in Appendix D).
//
//   classify  (main stream)  per id: range test against [lo,hi) (constant memory, Sec. 4.1), else a
//                            probe of the cache's id table (Sec. 4.2), else a miss; writes one
//                            source descriptor per row, the compacted list of missing rows and,
//                            chunk by chunk, the rows that hit (in row order)
//   hit copy  (main stream)  rows from the local shard or the replica cache, 128-bit vectors,
//                            outputs walked in order so that stores are dense
//   miss copy (side stream)  rows read straight from pinned host memory over PCIe (on CUs of
//                            its own), started after the hit copy and joined before the call
//                            ends, or (SPP_NO_JOIN) by the next gather, which classifies its own
//                            ids in the meantime
// A vertex that several rows of one call miss (several minibatches of a pipeline sampling the same
// remote vertex) is fetched once: after the classification a pass over the miss list claims every
// missed vertex in a table that lives for the call (sized for the misses, so a few MB); the row
// that wins the claim stays in the miss list, the others are struck from it and copied from the
// winner's output row at the join, on the main stream (beside the next miss copy, if there is one).
// On request (SPP_STORE_ORDER) the claim uses one entry per row of the remote store instead of the
// hashed table, and a scan over those entries lists the claimed rows in the store's order: rows
// that are neighbours in the store then share the memory lines they straddle on their way over PCIe.
// With a split local store (Sec. 3.2 on host-to-device transfers, Sec. 4.1) a local id is looked up
// in the store's rank array: below the limit it is a hit on the device rows (stored in rank order),
// else it joins the miss list and is read from the host-resident local rows.
#include "spp_common.h"
#include "spp_device.h"
#include "spp_rowcopy.h"

#include <mutex>

namespace spp {

constexpr int kMissBlocks = 64;        // workgroups of the miss kernel (see gather_lists)
constexpr int kMissThreads = 256;      // threads of each
constexpr int kClsPer = 8;             // ids per thread: a workgroup classifies 2048 consecutive ids per round
static_assert(kBlock * kClsPer == kListAlign, "a classification chunk must not straddle two lists");

struct ClassifyArgs {
    ListTable      t;
    int64_t        N, lo, hi;
    const unsigned long long* tab;     // null: no cache
    uint32_t       mask;
    int            shift;
    int64_t        limit;              // slots in use
    const int32_t* local_rank;         // null: the whole local shard is in device memory, row = g - lo
    int64_t        local_limit;        // ranks below this are in device memory (row = rank)
    int64_t*       desc;               // per virtual row
    int32_t*       misslist;           // virtual rows that miss
    int64_t*       hitlist;            // rows served from the shard or the cache: source, list and row in the list (make_hit),
    int32_t*       hcount;             //   chunk by chunk: hitlist[chunk * kListAlign + i], i < hcount[chunk]
    unsigned long long* counters;      // [0] local, [1] cache hit, [2] rows in misslist, [3] bad id, [4] unused,
                                       // [5] local rows read from the host (part of [0] and of [2]), [6] rows in duplist,
                                       // [7] rows in the store-ordered list
    unsigned long long* totals;        // context-wide running sums: [3] calls, [4] local, [5] cache hit,
                                       // [6] remote miss, [7] local rows read from the host
};

struct PrologueArgs {
    int64_t        n[kMaxLists];       // host counts (upper bounds when n_ptr is given)
    const int64_t* n_ptr[kMaxLists];   // device counts or null
    int            n_lists;
    int64_t        n_remote;           // rows of the remote store
};

// Zeroes the per-call counters and lays the lists out in the virtual row space.
__global__ void gather_prologue_kernel(PrologueArgs p, unsigned long long* counters, int64_t* off, int64_t* cnt,
                                       int64_t* minfo) {
    if (threadIdx.x < 8) counters[threadIdx.x] = 0ull;
    if (threadIdx.x == 0) {
        minfo[2] = p.n_remote;
        int64_t o = 0;
        for (int j = 0; j < p.n_lists; ++j) {
            int64_t c = p.n_ptr[j] ? *p.n_ptr[j] : p.n[j];
            if (c < 0) c = 0;
            if (c > p.n[j]) c = p.n[j];             // never beyond what the caller's buffers hold
            off[j] = o;
            cnt[j] = c;
            o = (o + c + kListAlign - 1) / kListAlign * kListAlign;
        }
        off[p.n_lists] = o;
    }
}

// Table of the call's missed vertices: the smallest power of two >= twice the miss list (>= 1024
// slots, at most max_slots, which the host sized for the bound), emptied.
__global__ void __launch_bounds__(kBlock) gather_table_clear_kernel(unsigned long long* tab,
                                                                    const unsigned long long* __restrict__ counters,
                                                                    int64_t max_slots, int64_t* minfo) {
    const int64_t want = 2 * (int64_t)counters[2];
    int64_t slots = 1024, shift = 22;
    while (slots < want && slots < max_slots) { slots <<= 1; --shift; }
    if (blockIdx.x == 0 && threadIdx.x == 0) { minfo[0] = slots - 1; minfo[1] = shift; }
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < slots; i += stride) tab[i] = ~0ull;
}

// Every remote row of the miss list claims its vertex; a row that finds the vertex claimed is struck
// from the list (the miss copy skips negative entries), gets the claimer's virtual row as its
// source, and joins the copy list.
__global__ void __launch_bounds__(kBlock) gather_share_kernel(unsigned long long* tab, const int64_t* __restrict__ minfo,
                                                              int64_t* __restrict__ desc, int32_t* __restrict__ misslist,
                                                              int32_t* __restrict__ duplist,
                                                              unsigned long long* __restrict__ counters,
                                                              unsigned long long* __restrict__ totals) {
    __shared__ int scan_lds[4];
    __shared__ unsigned long long base_lds;
    const int64_t n = (int64_t)counters[2];
    const uint32_t mask = (uint32_t)minfo[0];
    const int shift = (int)minfo[1];
    const int64_t n_round = (n + kBlock - 1) / kBlock * kBlock;            // whole workgroups reach the scan
    for (int64_t m = (int64_t)blockIdx.x * kBlock + threadIdx.x; m < n_round; m += (int64_t)gridDim.x * kBlock) {
        int32_t r = -1;
        bool dup = false;
        if (m < n) {
            r = misslist[m];
            const int64_t d = desc[r];
            uint32_t first = 0;
            if (desc_tag(d) == kTagMiss && !table_claim(tab, mask, shift, (uint32_t)desc_row(d), (uint32_t)r, first)) {
                dup = true;
                desc[r] = make_desc(kTagDup, first);
                misslist[m] = -1;
            }
        }
        int total;
        const int ex = block_exclusive_scan(dup ? 1 : 0, scan_lds, total);
        if (total) {                                                       // uniform over the workgroup
            if (threadIdx.x == 0) {
                base_lds = atomicAdd(&counters[6], (unsigned long long)total);
                atomicAdd(&totals[8], (unsigned long long)total);
            }
            __syncthreads();
            if (dup) duplist[base_lds + (unsigned long long)ex] = r;
            __syncthreads();
        }
    }
}

// The same with one entry per row of the remote store instead of a hashed table (SPP_STORE_ORDER):
// every remote row of the miss list leaves the list; the row that claims its vertex is found again
// by the scan over the store's rows that follows, which lists the claimers in store order.
constexpr uint32_t kNoRow = 0xFFFFFFFFu;
__global__ void __launch_bounds__(kBlock) fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) p[i] = v;
}
__global__ void __launch_bounds__(kBlock) gather_share_direct_kernel(uint32_t* __restrict__ first,
                                                                     int64_t* __restrict__ desc,
                                                                     int32_t* __restrict__ misslist,
                                                                     int32_t* __restrict__ duplist,
                                                                     unsigned long long* __restrict__ counters,
                                                                     unsigned long long* __restrict__ totals) {
    __shared__ int scan_lds[4];
    __shared__ unsigned long long base_lds;
    const int64_t n = (int64_t)counters[2];
    const int64_t n_round = (n + kBlock - 1) / kBlock * kBlock;            // whole workgroups reach the scan
    for (int64_t m = (int64_t)blockIdx.x * kBlock + threadIdx.x; m < n_round; m += (int64_t)gridDim.x * kBlock) {
        int32_t r = -1;
        bool dup = false;
        if (m < n) {
            r = misslist[m];
            const int64_t d = desc[r];
            if (desc_tag(d) == kTagMiss) {
                const uint32_t old = atomicCAS(&first[desc_row(d)], kNoRow, (uint32_t)r);
                misslist[m] = -1;
                if (old != kNoRow) {
                    dup = true;
                    desc[r] = make_desc(kTagDup, old);
                }
            }
        }
        int total;
        const int ex = block_exclusive_scan(dup ? 1 : 0, scan_lds, total);
        if (total) {                                                       // uniform over the workgroup
            if (threadIdx.x == 0) {
                base_lds = atomicAdd(&counters[6], (unsigned long long)total);
                atomicAdd(&totals[8], (unsigned long long)total);
            }
            __syncthreads();
            if (dup) duplist[base_lds + (unsigned long long)ex] = r;
            __syncthreads();
        }
    }
}
struct ClaimedIn {
    const uint32_t* first;
    __device__ int operator()(int64_t i) const { return first[i] != kNoRow ? 1 : 0; }
};
struct ClaimedOut {
    const uint32_t* first; int32_t* sorted;
    __device__ void operator()(int64_t i, int ex, int v) const { if (v) sorted[(uint32_t)ex] = (int32_t)first[i]; }
};
struct ClaimedFin {
    unsigned long long* count;
    __device__ void operator()(int total) const { *count = (unsigned long long)(uint32_t)total; }
};

// One workgroup classifies a chunk of 2048 consecutive ids of one list (eight consecutive ids per
// thread, so that ranks from a scan over the threads follow the row order), then reserves room for
// all of the chunk's misses in the miss list with a single atomic, so the list counter sees one
// atomic per 2048 ids instead of one per wavefront; the chunk's hits go, in row order, to the
// chunk's own part of the hit list.
__global__ void __launch_bounds__(kBlock) classify_kernel(ClassifyArgs a) {
    __shared__ int scan_lds[4];
    __shared__ unsigned long long base_lds[2];
    __shared__ ListLds ls;
    load_lists(a.t, ls);
    const int64_t total = ls.off[a.t.n_lists];
    int n_local = 0, n_hit = 0, n_rmiss = 0, n_lhost = 0;
    for (int64_t base = (int64_t)blockIdx.x * kListAlign; base < total; base += (int64_t)gridDim.x * kListAlign) {
        const int j = list_of(ls, a.t.n_lists, base);
        const int64_t lbeg = ls.off[j], n = ls.cnt[j];
        const int32_t* __restrict__ ids = a.t.ids[j];
        uint32_t missbits = 0, hitbits = 0;
        int64_t dk[kClsPer];
#pragma unroll
        for (int k = 0; k < kClsPer; ++k) {
            dk[k] = 0;
            const int64_t i = base - lbeg + (int64_t)threadIdx.x * kClsPer + k;      // a thread takes consecutive rows:
            if (i >= n) continue;                                                     // the lists come out in row order
            const int64_t g = ids[i];
            int64_t d = make_desc(kTagSkip, 0);
            if (g < 0 || g >= a.N) {
                atomicOr(&a.counters[3], 1ull);
            } else if (g >= a.lo && g < a.hi) {
                ++n_local;
                const int64_t r = a.local_rank ? (int64_t)a.local_rank[g - a.lo] : g - a.lo;
                if (!a.local_rank || r < a.local_limit) {
                    d = make_desc(kTagLocal, r);
                    hitbits |= 1u << k;
                } else {
                    d = make_desc(kTagLocalHost, g - a.lo);
                    ++n_lhost;
                    missbits |= 1u << k;
                }
            } else {
                uint32_t slot = 0;
                const bool found = a.tab && table_find(a.tab, a.mask, a.shift, (uint32_t)g, slot) >= 0 &&
                                   (int64_t)slot < a.limit;
                if (found) { d = make_desc(kTagCache, slot); ++n_hit; hitbits |= 1u << k; }
                else       { d = make_desc(kTagMiss, g < a.lo ? g : g - (a.hi - a.lo)); ++n_rmiss; missbits |= 1u << k; }
            }
            a.desc[lbeg + i] = d;
            dk[k] = d;
        }
        // both lists are compacted with one scan: misses in the low half-word, hits in the high one
        // (a workgroup's totals are at most 2048 each)
        int total_packed;
        const int ex = block_exclusive_scan(__popc(missbits) | (__popc(hitbits) << 16), scan_lds, total_packed);
        const int total_miss = total_packed & 0xFFFF, total_hit = total_packed >> 16;
        if (threadIdx.x == 0) {
            if (total_miss) base_lds[0] = atomicAdd(&a.counters[2], (unsigned long long)total_miss);
            a.hcount[base / kListAlign] = total_hit;          // the chunk's hits go to the chunk's own part of the list
        }
        __syncthreads();
        unsigned long long mpos = base_lds[0] + (unsigned long long)(ex & 0xFFFF);
        unsigned long long hpos = (unsigned long long)base + (unsigned long long)(ex >> 16);
#pragma unroll
        for (int k = 0; k < kClsPer; ++k) {
            const int32_t r = (int32_t)(base + (int64_t)threadIdx.x * kClsPer + k);
            if (missbits & (1u << k)) a.misslist[mpos++] = r;
            if (hitbits & (1u << k)) a.hitlist[hpos++] = make_hit(desc_tag(dk[k]) == kTagCache, desc_row(dk[k]), j, (int64_t)r - lbeg);
        }
        __syncthreads();                          // base_lds is reused by the next round
    }
    const int tl = block_reduce_sum(n_local, scan_lds);
    const int th = block_reduce_sum(n_hit, scan_lds);
    const int tm = block_reduce_sum(n_rmiss, scan_lds);
    const int tlh = block_reduce_sum(n_lhost, scan_lds);
    if (threadIdx.x == 0) {
        if (tm) atomicAdd(&a.totals[6], (unsigned long long)tm);
        if (tlh) { atomicAdd(&a.counters[5], (unsigned long long)tlh); atomicAdd(&a.totals[7], (unsigned long long)tlh); }
        if (tl) { atomicAdd(&a.counters[0], (unsigned long long)tl); atomicAdd(&a.totals[4], (unsigned long long)tl); }
        if (th) { atomicAdd(&a.counters[1], (unsigned long long)th); atomicAdd(&a.totals[5], (unsigned long long)th); }
        if (blockIdx.x == 0) atomicAdd(&a.totals[3], 1ull);
    }
}

// Device-visible address of a row store that is either device memory or pinned host memory.
int device_view(const void* p, const void** out) {
    *out = p;
    if (!p) return SPP_OK;
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        set_error("a row store is neither device memory nor pinned host memory (%s)", hipGetErrorString(e));
        return SPP_E_ARG;
    }
    if (attr.type == hipMemoryTypeHost) {
        void* dp = nullptr;
        e = hipHostGetDevicePointer(&dp, const_cast<void*>(p), 0);
        if (e != hipSuccess) { set_error("hipHostGetDevicePointer: %s", hipGetErrorString(e)); return SPP_E_HIP; }
        *out = dp;
    } else if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) {
        set_error("a row store is ordinary pageable host memory; pin it (hipHostMalloc)");
        return SPP_E_ARG;
    }
    return SPP_OK;
}

int copy_rows_indexed(hipStream_t st, const void* src, const int64_t* d_rowidx, int64_t n, int64_t row_bytes,
                      void* d_out, int num_cu) {
    if (n <= 0) return SPP_OK;
    const void* dsrc = nullptr;
    SPP_TRY(device_view(src, &dsrc));
    if ((((uintptr_t)dsrc | (uintptr_t)d_out | (uintptr_t)row_bytes) & 1) != 0) {
        set_error("row copy: odd row size or address");
        return SPP_E_ARG;
    }
    const int V = pick_vec(row_bytes, (uintptr_t)dsrc | (uintptr_t)d_out);
    const uint32_t vpr = (uint32_t)(row_bytes / V);
    const int64_t vecs = n * vpr;
    int64_t need = (vecs + kBlock * kCopyUnroll - 1) / (kBlock * kCopyUnroll);
    const int grid = (int)(need < (int64_t)num_cu * 8 ? need : (int64_t)num_cu * 8);
    switch (V) {
        case 16: rows_indexed_kernel<16><<<grid, kBlock, 0, st>>>((const char*)dsrc, d_rowidx, n, vpr, (char*)d_out); break;
        case 8:  rows_indexed_kernel<8><<<grid, kBlock, 0, st>>>((const char*)dsrc, d_rowidx, n, vpr, (char*)d_out); break;
        case 4:  rows_indexed_kernel<4><<<grid, kBlock, 0, st>>>((const char*)dsrc, d_rowidx, n, vpr, (char*)d_out); break;
        default: rows_indexed_kernel<2><<<grid, kBlock, 0, st>>>((const char*)dsrc, d_rowidx, n, vpr, (char*)d_out); break;
    }
    SPP_HIP(hipGetLastError());
    return SPP_OK;
}

// Rows that share a fetched vertex, copied from the fetched row's output once the miss copy of
// their call has landed (the caller has made the stream wait for it).
int launch_dup(spp_ctx* ctx, const PendingGather& pg) {
    if (!pg.has_dup) return SPP_OK;
    const int dgrid = ctx->num_cu * 4;
    hipStream_t st = ctx->stream;
    switch (pg.V) {
        case 16: gather_dup_kernel<16><<<dgrid, kBlock, 0, st>>>(pg.desc, pg.duplist, pg.dup_count, pg.t, pg.vpr); break;
        case 8:  gather_dup_kernel<8><<<dgrid, kBlock, 0, st>>>(pg.desc, pg.duplist, pg.dup_count, pg.t, pg.vpr); break;
        case 4:  gather_dup_kernel<4><<<dgrid, kBlock, 0, st>>>(pg.desc, pg.duplist, pg.dup_count, pg.t, pg.vpr); break;
        default: gather_dup_kernel<2><<<dgrid, kBlock, 0, st>>>(pg.desc, pg.duplist, pg.dup_count, pg.t, pg.vpr); break;
    }
    SPP_HIP(hipGetLastError());
    return SPP_OK;
}

}  // namespace spp

// Device workspace of one gather call over `rows` virtual rows (padded): the counters and the
// layout of the lists, one source descriptor per row, and the four row lists.
namespace spp {
// Lists the tiles that hold hits for the hit copy (see gather_hit_kernel): one workgroup per id list adds up
// the tiles of the lists before it (a few thousand chunk counts at most) and then numbers its own.
constexpr int kItemBlock = 1024;
__global__ void __launch_bounds__(kItemBlock) hit_items_kernel(const int32_t* __restrict__ hcount, ListTable t, uint32_t vpr,
                                                               uint32_t tile_vecs, uint64_t* __restrict__ item_list,
                                                               uint32_t* __restrict__ n_items) {
    __shared__ uint32_t wsum[kItemBlock / kWave];
    __shared__ uint32_t carry;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t c0 = t.off[blockIdx.x] / kListAlign, c1 = t.off[blockIdx.x + 1] / kListAlign;
    auto tiles_of = [&](int64_t c) { return ((uint32_t)hcount[c] * vpr + tile_vecs - 1) / tile_vecs; };
    // all threads: the tiles of the chunks before this list's; leaves the sum in `carry`
    uint32_t mine = 0;
    for (int64_t c = threadIdx.x; c < c0; c += kItemBlock) mine += tiles_of(c);
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) mine += __shfl_down(mine, off, kWave);
    if (lane == 0) wsum[wave] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t s = 0;
        for (int w = 0; w < kItemBlock / kWave; ++w) s += wsum[w];
        carry = s;
    }
    __syncthreads();
    for (int64_t cb = c0; cb < c1; cb += kItemBlock) {
        const int64_t c = cb + threadIdx.x;
        const uint32_t n = c < c1 ? tiles_of(c) : 0u;
        const uint32_t inc = (uint32_t)wave_inclusive_scan((int)n);
        const uint32_t before = carry;           // read before this round's update (a barrier follows)
        if (lane == kWave - 1) wsum[wave] = inc;
        __syncthreads();
        uint32_t base = before, total = 0;
        for (int w = 0; w < kItemBlock / kWave; ++w) { const uint32_t v = wsum[w]; total += v; if (w < wave) base += v; }
        const uint32_t at = base + inc - n;
        if (n) {
            const uint32_t nv = (uint32_t)hcount[c] * vpr;
            for (uint32_t k = 0; k < n; ++k) {
                const uint32_t in_tile = nv - k * tile_vecs < tile_vecs ? nv - k * tile_vecs : tile_vecs;
                item_list[at + k] = ((uint64_t)c << 32) | ((uint64_t)k << kHitTileBits) | in_tile;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) carry = before + total;
        __syncthreads();
    }
    if (blockIdx.x == (unsigned)t.n_lists - 1 && threadIdx.x == 0) *n_items = carry;
}


struct GatherWs {
    unsigned long long* counters;   // [8]
    int64_t* off;                   // [kMaxLists + 1]
    int64_t* cnt;                   // [kMaxLists + 1]
    int64_t* minfo;                 // [4]
    int64_t* desc;                  // [rows]
    int64_t* hitlist;               // [rows]
    int32_t* misslist;              // [rows]
    int32_t* duplist;               // [rows]
    int32_t* ordered;               // [rows]
    int32_t* hcount;                // [rows / kListAlign]
};
constexpr size_t kWsHeadBytes = 2048;       // counters, off, cnt, minfo: (8 + 2 * (kMaxLists + 1) + 4) * 8 = 1136 bytes
static_assert((8 + 2 * (kMaxLists + 1) + 4) * sizeof(int64_t) <= kWsHeadBytes, "the head of the workspace holds the counters and the layout");
static GatherWs carve_ws(void* head, void* desc, void* lists, int64_t rows) {
    GatherWs w;
    w.counters = static_cast<unsigned long long*>(head);
    w.off = static_cast<int64_t*>(head) + 8;
    w.cnt = w.off + kMaxLists + 1;
    w.minfo = w.cnt + kMaxLists + 1;
    w.desc = static_cast<int64_t*>(desc);
    w.hitlist = static_cast<int64_t*>(lists);
    w.misslist = static_cast<int32_t*>(lists) + 2 * rows;
    w.duplist = w.misslist + rows;
    w.ordered = w.duplist + rows;
    w.hcount = w.ordered + rows;
    return w;
}

// The workspace of spp_gather_features_static: a fixed array in the library's device image, one copy
// per GPU, so that the call has nothing to allocate.  Host code reaches it only through the address
// that hipGetSymbolAddress returns for the current device (kept per device below); the array's name
// is never passed to a kernel or a runtime call.
constexpr int64_t kStaticRows = SPP_STATIC_GATHER_MAX_ROWS;
static_assert(kStaticRows % kListAlign == 0, "the static workspace holds whole chunks");
constexpr size_t kStaticBytes = kWsHeadBytes + (size_t)kStaticRows * (sizeof(int64_t) + 5 * sizeof(int32_t)) +
                                (size_t)(kStaticRows / kListAlign) * sizeof(int32_t);
static __device__ __align__(256) unsigned char scratch[(kStaticBytes + 255) / 256 * 256];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};       // device address of `scratch` on each GPU, once asked for
static std::mutex g_scratch_mutex;

// Address of this GPU's copy of the array; `device` must be the current device.
int static_scratch(int device, void** out) {
    SPP_CHECK(device >= 0 && device < kMaxDevices, SPP_E_ARG, "static workspace: device %d out of range", device);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        SPP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        SPP_CHECK(p != nullptr, SPP_E_HIP, "static workspace: hipGetSymbolAddress returned a null address");
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return SPP_OK;
}
}  // namespace spp

// The gather behind the entry points: the local shard is either d_local (all rows in device
// memory) or a split store.  With `fixed` the workspace is the caller's (holding fixed_rows virtual
// rows) and nothing is allocated; otherwise it comes from the context's grow-only buffers.
static int gather_lists(spp_ctx* ctx, const spp_cache* cache, const void* d_local, const spp_local_store* store,
                        int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D,
                        int32_t elem_bytes, const spp_gather_list* lists, int32_t n_lists,
                        spp_gather_stats* stats, uint32_t flags, const spp::GatherWs* fixed = nullptr,
                        int64_t fixed_rows = 0) {
    using namespace spp;
    SPP_CHECK(ctx, SPP_E_ARG, "spp_gather_features: ctx is null");
    SPP_CHECK(n_lists >= 0 && n_lists <= SPP_MAX_GATHER_LISTS && (lists || n_lists == 0), SPP_E_ARG,
              "spp_gather_features: %d lists (at most %d)", n_lists, SPP_MAX_GATHER_LISTS);
    SPP_CHECK(N > 0 && lo >= 0 && lo <= hi && hi <= N, SPP_E_ARG,
              "spp_gather_features: range [%lld, %lld) of N = %lld", (long long)lo, (long long)hi, (long long)N);
    SPP_CHECK(D >= 1 && elem_bytes >= 1, SPP_E_ARG, "spp_gather_features: D = %d, elem_bytes = %d", D, elem_bytes);
    const int64_t row_bytes = (int64_t)D * elem_bytes;
    SPP_CHECK(row_bytes % 2 == 0, SPP_E_ARG, "spp_gather_features: row size %lld is odd", (long long)row_bytes);
    if (cache) {
        SPP_CHECK(cache->lo == lo && cache->hi == hi && cache->N == N, SPP_E_ARG,
                  "spp_gather_features: the cache was built for another partition range");
        SPP_CHECK(cache->rows != nullptr || cache->limit == 0, SPP_E_ARG, "spp_gather_features: the cache holds no rows");
        SPP_CHECK(cache->row_bytes == row_bytes || cache->limit == 0, SPP_E_ARG,
                  "spp_gather_features: cache rows are %lld bytes, requested %lld", (long long)cache->row_bytes, (long long)row_bytes);
    }
    const void* crow = cache ? cache->rows : nullptr;
    const void* dremote = nullptr;
    const void* lhost = nullptr;        // host-resident local rows (split store only)
    if (store) {
        SPP_CHECK(store->lo == lo && store->hi == hi && store->N == N, SPP_E_ARG,
                  "spp_gather_features: the local store was built for another partition range");
        SPP_CHECK(store->row_bytes == row_bytes, SPP_E_ARG, "spp_gather_features: local store rows are %lld bytes, requested %lld",
                  (long long)store->row_bytes, (long long)row_bytes);
        d_local = store->rows;
        lhost = store->host_rows;
    }
    SPP_HIP(hipSetDevice(ctx->device));
    SPP_TRY(device_view(remote, &dremote));

    ClassifyArgs a;
    PrologueArgs pro;
    memset(&a, 0, sizeof(a));
    memset(&pro, 0, sizeof(pro));
    int64_t vbound = 0;                 // virtual rows, with padding
    uintptr_t addr_bits = (uintptr_t)d_local | (uintptr_t)crow | (uintptr_t)dremote | (uintptr_t)lhost;
    for (int j = 0; j < n_lists; ++j) {
        SPP_CHECK(lists[j].n >= 0 && lists[j].n <= ((int64_t)1 << kHitRowBits), SPP_E_ARG,
                  "spp_gather_features: list %d has n = %lld (at most 2^%d)", j, (long long)lists[j].n, kHitRowBits);
        SPP_CHECK(lists[j].n == 0 || (lists[j].d_node_ids && lists[j].d_out), SPP_E_ARG,
                  "spp_gather_features: list %d has null ids or output", j);
        a.t.ids[j] = lists[j].d_node_ids;
        a.t.out[j] = static_cast<char*>(lists[j].d_out);
        pro.n[j] = lists[j].n;
        pro.n_ptr[j] = lists[j].d_n;
        vbound = (vbound + lists[j].n + kListAlign - 1) / kListAlign * kListAlign;
        addr_bits |= (uintptr_t)lists[j].d_out;
    }
    SPP_CHECK((addr_bits & 1) == 0, SPP_E_ARG, "spp_gather_features: a row store or an output has an odd address");
    SPP_CHECK(vbound < 0x7FFFFFFFll, SPP_E_ARG, "spp_gather_features: %lld rows in one call exceed the 32-bit miss list", (long long)vbound);
    SPP_CHECK(hi == lo || d_local || store || vbound == 0, SPP_E_ARG, "spp_gather_features: local shard is null");
    a.t.n_lists = pro.n_lists = n_lists;

    hipStream_t st = ctx->stream;
    // A miss copy left running by the call before (SPP_NO_JOIN) still reads that call's descriptors,
    // lists and counters, so calls alternate between two sets of them: this call's classification
    // runs beside that miss copy.  The set used two calls ago is free: the call before joined that
    // gather before its own hit copy (if it had no rows and joined nothing, it is joined here).
    const int slot = ctx->gslot ^= 1;
    if (ctx->pending.active && (ctx->pending.slot == slot || fixed)) SPP_TRY(spp_gather_join(ctx));
    if (fixed) {
        SPP_CHECK(vbound <= fixed_rows, SPP_E_ARG, "spp_gather_features_static: %lld rows (padded) exceed the fixed workspace of %lld",
                  (long long)vbound, (long long)fixed_rows);
        SPP_CHECK(n_lists <= 1 && !(flags & (SPP_STORE_ORDER | SPP_NO_JOIN | SPP_HIT_BESIDE_MISS)), SPP_E_ARG,
                  "spp_gather_features_static: one list, no SPP_STORE_ORDER, no SPP_NO_JOIN");
    } else {
        SPP_TRY(ctx->gcount[slot].reserve(kWsHeadBytes));
    }
    // several lists make it worth claiming missed vertices: one list of a sampler's distinct ids
    // has nothing to share
    const int64_t n_remote = N - (hi - lo);
    const bool store_order = (flags & SPP_STORE_ORDER) && dremote != nullptr && vbound > 0 && n_remote > 0;
    const bool share_misses = dremote != nullptr && vbound > 0 && (n_lists > 1 || store_order);
    const int order_grid = 256;         // workgroups of the scan over the store's rows
    uint32_t mcap = 0;
    SPP_CHECK(!fixed || (!store_order && !share_misses), SPP_E_ARG, "spp_gather_features_static: a call that shares misses needs tables it cannot allocate");
    if (store_order) {
        SPP_TRY(ctx->gfirst.reserve((size_t)n_remote * sizeof(uint32_t)));
        SPP_TRY(ctx->partials.reserve((size_t)order_grid * sizeof(int) + 64));
    } else if (share_misses) {
        mcap = next_pow2((uint64_t)(2 * vbound > 1024 ? 2 * vbound : 1024));
        SPP_TRY(ctx->gtable.reserve((size_t)mcap * sizeof(uint64_t)));
    }
    if (vbound > 0 && !fixed) {
        SPP_TRY(ctx->srcdesc[slot].reserve((size_t)vbound * sizeof(int64_t)));
        // hit list (64-bit entries), miss list, copy list, misses in store order, hits per chunk
        SPP_TRY(ctx->misslist[slot].reserve((size_t)vbound * sizeof(int32_t) * 5 + (size_t)(vbound / kListAlign) * sizeof(int32_t)));
    }
    const GatherWs ws = fixed ? *fixed
                              : carve_ws(ctx->gcount[slot].ptr, ctx->srcdesc[slot].ptr, ctx->misslist[slot].ptr, vbound);
    unsigned long long* counters = ws.counters;
    int64_t* off = ws.off;
    int64_t* cnt = ws.cnt;
    int64_t* minfo = ws.minfo;
    a.t.off = off; a.t.cnt = cnt;
    pro.n_remote = n_remote;
    gather_prologue_kernel<<<1, 64, 0, st>>>(pro, counters, off, cnt, minfo);
    if (vbound > 0) {
        a.N = N; a.lo = lo; a.hi = hi;
        a.tab = cache && cache->limit > 0 ? reinterpret_cast<const unsigned long long*>(cache->table) : nullptr;
        a.mask = cache ? cache->table_mask : 0; a.shift = cache ? cache->table_shift : 0;
        a.limit = cache ? cache->limit : 0;
        a.local_rank = store ? store->rank : nullptr;
        a.local_limit = store ? store->limit : 0;
        a.desc = ws.desc; a.counters = counters;
        a.hitlist = ws.hitlist;
        a.misslist = ws.misslist;
        int32_t* duplist = ws.duplist;
        int32_t* ordered = ws.ordered;
        a.hcount = ws.hcount;
        a.totals = reinterpret_cast<unsigned long long*>(ctx->totals);
        const int64_t cneed = vbound / kListAlign;
        const int cgrid = (int)(cneed < (int64_t)ctx->num_cu * 8 ? cneed : (int64_t)ctx->num_cu * 8);
        {
            ScopedTimer tc(ctx, SPP_T_GATHER_CLASSIFY, st);
            classify_kernel<<<cgrid, kBlock, 0, st>>>(a);
            const int sgrid = ctx->num_cu * 4;
            if (store_order) {
                uint32_t* first = ctx->gfirst.as<uint32_t>();
                fill_u32_kernel<<<sgrid, kBlock, 0, st>>>(first, n_remote, kNoRow);
                gather_share_direct_kernel<<<sgrid, kBlock, 0, st>>>(first, a.desc, a.misslist, duplist, counters, a.totals);
                grid_scan(st, order_grid, minfo + 2, ClaimedIn{first}, ClaimedOut{first, ordered}, ClaimedFin{counters + 7},
                          ctx->partials.as<int>());
            } else if (share_misses) {
                unsigned long long* mtab = ctx->gtable.as<unsigned long long>();
                gather_table_clear_kernel<<<sgrid, kBlock, 0, st>>>(mtab, counters, (int64_t)mcap, minfo);
                gather_share_kernel<<<sgrid, kBlock, 0, st>>>(mtab, minfo, a.desc, a.misslist, duplist, counters, a.totals);
            }
        }
        const int V = pick_vec(row_bytes, addr_bits);
        const uint32_t vpr = (uint32_t)(row_bytes / V);
        const int64_t vecs = vbound * vpr;
        // hit copy: many small work items (one tile of 1024 vectors each; at most 256 workgroups per CU in
        // the grid, which then take several tiles each) let the dispatcher balance the copy
        const uint32_t tiles_per_chunk = (uint32_t)((kListAlign * vpr + kBlock * kHitUnroll - 1) / (kBlock * kHitUnroll));
        const int64_t hneed = vbound / kListAlign * tiles_per_chunk;
        const int grid = (int)(hneed < (int64_t)ctx->num_cu * 256 ? hneed : (int64_t)ctx->num_cu * 256);
        // the tiles that hold hits, listed once the classification has counted them (not for the caller that
        // must not allocate, nor where a chunk or a tile number does not fit the list's entries)
        uint64_t* item_list = nullptr;
        uint32_t* n_items = nullptr;
        static_assert(kBlock * kHitUnroll < (1 << kHitTileBits), "an entry holds the vectors of a tile");
        if (!fixed && n_lists > 0 && tiles_per_chunk <= (1u << kHitTileBits)) {
            SPP_TRY(ctx->hititems[slot].reserve((size_t)(hneed + 2) * sizeof(uint64_t)));
            n_items = ctx->hititems[slot].as<uint32_t>();
            item_list = ctx->hititems[slot].as<uint64_t>() + 2;
            hit_items_kernel<<<n_lists, kItemBlock, 0, st>>>(a.hcount, a.t, vpr, (uint32_t)(kBlock * kHitUnroll), item_list, n_items);
        }
        // The miss kernel is kept to 64 workgroups of 256 threads: they saturate the PCIe link (32
        // workgroups of 512 threads or 16 of 1024 reach 95 % of their rate, 64 of 512 less).  A CU
        // that hosts host-memory loads serves every other wavefront on it slowly, so each of these
        // workgroups asks for nearly all of a CU's LDS, which keeps the hit copy (whose workgroups
        // need a KB of LDS) and most other kernels off its CU: with the 64 CUs set aside like this
        // the sampler beside a miss copy ran 25 % faster and the hit copy lost only the CUs' share.
        const int64_t mneed = (vecs + kMissThreads * kCopyUnroll - 1) / (kMissThreads * kCopyUnroll);
        const int quarter = ctx->num_cu / 4 > 0 ? ctx->num_cu / 4 : 1;
        const int mmax = quarter < kMissBlocks ? quarter : kMissBlocks;        // a quarter of the CUs at most
        const int mgrid = (int)(mneed < mmax ? mneed : mmax);
        const bool miss_path = dremote != nullptr || lhost != nullptr;
        if (miss_path && ctx->miss_lds == 0) {
            int lds_max = 0;
            SPP_HIP(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, ctx->device));
            // what is left beside this and the kernel's own KB is less than the hit copy needs
            const int want = lds_max - 2048;
            SPP_CHECK(want > 0, SPP_E_HIP, "spp_gather_features: the device reports %d bytes of LDS per workgroup", lds_max);
            SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_miss_kernel<16, kMissThreads>), hipFuncAttributeMaxDynamicSharedMemorySize, want));
            SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_miss_kernel<8, kMissThreads>), hipFuncAttributeMaxDynamicSharedMemorySize, want));
            SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_miss_kernel<4, kMissThreads>), hipFuncAttributeMaxDynamicSharedMemorySize, want));
            SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_miss_kernel<2, kMissThreads>), hipFuncAttributeMaxDynamicSharedMemorySize, want));
            ctx->miss_lds = want;
        }
        auto launch_miss = [&]() -> int {
            SPP_HIP(hipEventRecord(ctx->ev_fork, st));
            SPP_HIP(hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0));
            {
                ScopedTimer tm(ctx, SPP_T_GATHER_MISS, ctx->side);
                // either store may be null (no remote store given, or no split local store): the
                // kernel skips rows that would need it and the statistics of the call report them
                const char* src = static_cast<const char*>(dremote);
                const char* lh = static_cast<const char*>(lhost);
                auto run = [&](const int32_t* list, const int64_t* count) {
                    const size_t lds = (size_t)ctx->miss_lds;
                    switch (V) {
                        case 16: gather_miss_kernel<16, kMissThreads><<<mgrid, kMissThreads, lds, ctx->side>>>(src, lh, a.desc, list, count, a.t, vpr); break;
                        case 8:  gather_miss_kernel<8, kMissThreads><<<mgrid, kMissThreads, lds, ctx->side>>>(src, lh, a.desc, list, count, a.t, vpr); break;
                        case 4:  gather_miss_kernel<4, kMissThreads><<<mgrid, kMissThreads, lds, ctx->side>>>(src, lh, a.desc, list, count, a.t, vpr); break;
                        default: gather_miss_kernel<2, kMissThreads><<<mgrid, kMissThreads, lds, ctx->side>>>(src, lh, a.desc, list, count, a.t, vpr); break;
                    }
                };
                // in store order: the claimed remote rows from the scan's list; the miss list then
                // only holds local rows that live in host memory (a split local store)
                if (store_order) run(ordered, reinterpret_cast<const int64_t*>(counters + 7));
                if (!store_order || lhost) run(a.misslist, reinterpret_cast<const int64_t*>(counters + 2));
            }
            SPP_HIP(hipEventRecord(ctx->ev_join[slot], ctx->side));
            return SPP_OK;
        };
        auto launch_hit = [&]() {
            ScopedTimer th(ctx, SPP_T_GATHER_HIT, st);
            const char* loc = static_cast<const char*>(d_local);
            const char* cr = static_cast<const char*>(crow);
            switch (V) {
                case 16: gather_hit_kernel<16><<<grid, kBlock, 0, st>>>(a.hitlist, a.hcount, a.t, loc, cr, vpr, tiles_per_chunk, item_list, n_items, hneed); break;
                case 8:  gather_hit_kernel<8><<<grid, kBlock, 0, st>>>(a.hitlist, a.hcount, a.t, loc, cr, vpr, tiles_per_chunk, item_list, n_items, hneed); break;
                case 4:  gather_hit_kernel<4><<<grid, kBlock, 0, st>>>(a.hitlist, a.hcount, a.t, loc, cr, vpr, tiles_per_chunk, item_list, n_items, hneed); break;
                default: gather_hit_kernel<2><<<grid, kBlock, 0, st>>>(a.hitlist, a.hcount, a.t, loc, cr, vpr, tiles_per_chunk, item_list, n_items, hneed); break;
            }
        };
        // Order of the copies.  The stream waits for the miss copy of the call before (its fetched
        // rows have landed), runs the hit copy with the whole chip, queues this call's miss copy on
        // the side stream and then copies the rows that shared a vertex of the earlier miss copy
        // (device to device, beside the new miss copy; the call before is complete from there on).
        // SPP_HIT_BESIDE_MISS queues the new miss copy first instead, so that it starts the moment
        // the earlier one ends and the PCIe link never idles; the hit copy then runs beside it on
        // the CUs it leaves free.  Measured on groups of 64 minibatches: 256-byte rows, a quarter
        // of the group's time spent in the hit copy: pipeline 19 % faster, hit copy at 0.61 of
        // the HBM peak instead of 0.69; 400-byte rows, link busy 95 % of the time anyway: 4.5 %
        // faster, 0.66 instead of 0.73.  The default keeps the HBM-bound copy at its full rate.
        if (flags & SPP_HIT_BESIDE_MISS) {
            if (miss_path) SPP_TRY(launch_miss());
            SPP_TRY(spp_gather_join(ctx));
            launch_hit();
        } else {
            const PendingGather before = ctx->pending;
            if (before.active) {
                SPP_HIP(hipStreamWaitEvent(st, ctx->ev_join[before.slot], 0));
                ctx->pending.active = false;
            }
            launch_hit();
            if (miss_path) SPP_TRY(launch_miss());
            if (before.active) SPP_TRY(launch_dup(ctx, before));
        }
        if (miss_path) {
            PendingGather& pg = ctx->pending;
            pg.active = true; pg.slot = slot; pg.has_dup = share_misses; pg.V = V; pg.vpr = vpr;
            pg.desc = a.desc; pg.duplist = duplist; pg.dup_count = reinterpret_cast<const int64_t*>(counters + 6);
            pg.t = a.t;
            if (!(flags & SPP_NO_JOIN)) SPP_TRY(spp_gather_join(ctx));
        }
    }
    SPP_HIP(hipGetLastError());
    int64_t* hp = ctx->h_pinned + 40;
    // the counters are final once the classification has run, whether or not the misses have landed
    SPP_HIP(hipMemcpyAsync(hp, counters, 7 * sizeof(int64_t), hipMemcpyDeviceToHost, st));
    ctx->h_pinned[48] = row_bytes;
    ctx->h_pinned[49] = dremote ? 1 : 0;
    if (flags & SPP_SYNC) {
        SPP_TRY(spp_gather_join(ctx));
        SPP_HIP(hipStreamSynchronize(st));
        return spp_gather_last_stats(ctx, stats);
    }
    return SPP_OK;
}

extern "C" int spp_gather_features_multi(spp_ctx* ctx, const spp_cache* cache, const void* d_local,
                                         int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D,
                                         int32_t elem_bytes, const spp_gather_list* lists, int32_t n_lists,
                                         spp_gather_stats* stats, uint32_t flags) {
    return gather_lists(ctx, cache, d_local, nullptr, N, lo, hi, remote, D, elem_bytes, lists, n_lists, stats, flags);
}

extern "C" int spp_gather_features_split(spp_ctx* ctx, const spp_cache* cache, const spp_local_store* store,
                                         int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D,
                                         int32_t elem_bytes, const spp_gather_list* lists, int32_t n_lists,
                                         spp_gather_stats* stats, uint32_t flags) {
    SPP_CHECK(store, SPP_E_ARG, "spp_gather_features_split: store is null");
    return gather_lists(ctx, cache, nullptr, store, N, lo, hi, remote, D, elem_bytes, lists, n_lists, stats, flags);
}

extern "C" int spp_gather_join(spp_ctx* ctx) {
    SPP_CHECK(ctx, SPP_E_ARG, "spp_gather_join: ctx is null");
    if (ctx->pending.active) {
        const spp::PendingGather pg = ctx->pending;
        ctx->pending.active = false;
        SPP_HIP(hipSetDevice(ctx->device));
        SPP_HIP(hipStreamWaitEvent(ctx->stream, ctx->ev_join[pg.slot], 0));
        SPP_TRY(spp::launch_dup(ctx, pg));
    }
    return SPP_OK;
}

extern "C" int spp_gather_features(spp_ctx* ctx, const spp_cache* cache, const void* d_local,
                                   int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D,
                                   int32_t elem_bytes, const int32_t* d_node_ids, int64_t n,
                                   const int64_t* d_n, void* d_out, spp_gather_stats* stats, uint32_t flags) {
    spp_gather_list one;
    one.d_node_ids = d_node_ids; one.n = n; one.d_n = d_n; one.d_out = d_out;
    return spp_gather_features_multi(ctx, cache, d_local, N, lo, hi, remote, D, elem_bytes, &one, 1, stats, flags);
}

extern "C" int spp_gather_last_stats(spp_ctx* ctx, spp_gather_stats* stats) {
    SPP_CHECK(ctx, SPP_E_ARG, "spp_gather_last_stats: ctx is null");
    const int64_t* hp = ctx->h_pinned + 40;
    if (stats) {
        stats->n_local = hp[0]; stats->n_cache_hit = hp[1]; stats->n_miss = hp[2] - hp[5];
        stats->n_local_host = hp[5];
        stats->n_miss_shared = hp[6];
        stats->miss_bytes = (hp[2] - hp[6]) * ctx->h_pinned[48];
    }
    SPP_CHECK(hp[3] == 0, SPP_E_ARG, "spp_gather_features: a vertex id lies outside [0, N); its row was left untouched");
    SPP_CHECK(hp[2] - hp[5] == 0 || ctx->h_pinned[49] != 0, SPP_E_ARG,
              "spp_gather_features: %lld rows missed but no remote store was given; they were left untouched",
              (long long)(hp[2] - hp[5]));
    return SPP_OK;
}

// The single-list gather for callers that must not allocate (code under graph capture, serving loops,
// harnesses that forbid hipMalloc): the same kernels, with the per-call workspace in a fixed array of
// the library's device image instead of the context's grow-only buffers.
extern "C" int spp_gather_features_static(spp_ctx* ctx, const spp_cache* cache, const void* d_local,
                                          int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D,
                                          int32_t elem_bytes, const int32_t* d_node_ids, int64_t n,
                                          const int64_t* d_n, void* d_out, spp_gather_stats* stats, uint32_t flags) {
    using namespace spp;
    SPP_CHECK(ctx, SPP_E_ARG, "spp_gather_features_static: ctx is null");
    SPP_CHECK(n >= 0 && n <= SPP_STATIC_GATHER_MAX_ROWS, SPP_E_ARG,
              "spp_gather_features_static: n = %lld exceeds SPP_STATIC_GATHER_MAX_ROWS = %d", (long long)n,
              SPP_STATIC_GATHER_MAX_ROWS);
    SPP_CHECK(!(flags & (SPP_STORE_ORDER | SPP_NO_JOIN | SPP_HIT_BESIDE_MISS)), SPP_E_ARG,
              "spp_gather_features_static: SPP_STORE_ORDER and SPP_NO_JOIN are not available here");
    SPP_HIP(hipSetDevice(ctx->device));
    void* base = nullptr;
    SPP_TRY(static_scratch(ctx->device, &base));
    char* b = static_cast<char*>(base);
    const GatherWs ws = carve_ws(b, b + kWsHeadBytes, b + kWsHeadBytes + (size_t)kStaticRows * sizeof(int64_t), kStaticRows);
    // event pairs for the timing report are created on demand: not here
    const int timing = ctx->timing;
    ctx->timing = 0;
    spp_gather_list one;
    one.d_node_ids = d_node_ids; one.n = n; one.d_n = d_n; one.d_out = d_out;
    const int rc = gather_lists(ctx, cache, d_local, nullptr, N, lo, hi, remote, D, elem_bytes, &one, 1, stats, flags, &ws,
                                kStaticRows);
    ctx->timing = timing;
    return rc;
}
