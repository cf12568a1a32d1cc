// Node-wise fanout sampling into per-layer message-flow graphs (Sec. 2.3; the process of Sec. 3.1).
//
// Up to 64 minibatches are sampled by one set of launches: every kernel has a second grid dimension
// that names the minibatch, and each minibatch has its own id table, flat-id buffer and counts, so
// the minibatches never interact.  Per hop h, all on the context's stream with every count kept on
// the device:
//   1. grid scan of c_i = min(f_h, d(S_{h-1}[i]))            -> indptr of MFG h, e_h
//   2. sample: a group of G lanes (G = 8/16/32/64 >= f_h) per target draws its slots in parallel
//      (one Philox block per lane), resolves Floyd's "already taken" rule with ballots, reads the
//      neighbour ids and stores them in flat (edge) order
//   3. dedup: for every sampled id the position of its first appearance among S_{h-1} followed by
//      the hop's flat list (an index below n_{h-1} means the vertex is an earlier one)
//   4. grid scan of "this flat entry is the first appearance of a new id"
//                                                            -> S_h appended in order, n_h, src of those entries
//   5. relabel: src[e] of a repeated id = its index in S_{h-1}, or the src of its first appearance
// Step 3 is where the ids meet.  A hop of up to 16 x 8192 ids (with S_{h-1}) is deduplicated in LDS:
// the ids are dealt by hash to up to 16 partitions, one workgroup per partition keeps an id table of
// 16384 slots in LDS (128 KB), reads the minibatch's whole list (a few hundred KB, from L2), inserts
// the ids of its partition with LDS atomics (smallest position wins) and, after a barrier, writes
// out what each of them resolved to.  Global memory sees only sequential reads and writes.  (The
// earlier form, a table in global memory fed by the sample kernel, was bound by the rate of global
// atomics, about 16 G/s: 0.31 ms for the 5 M inserts of the last hop of 64 minibatches.)  Larger hops
// keep that form: the id table (open addressing, global memory) is right-sized per hop on the device:
// once e_h is known, the hop uses the first 2^k >= 2 (n_{h-1} + e_h) slots of the minibatch's region,
// clears exactly those, and the sample kernel offers S_{h-1} (value = index, which is below any
// position offered at this hop, so earlier vertices keep their ids) next to the new ids with atomic
// minima; the scan's first pass then reads what each entry resolved to.  The worst-case bound on
// |S_L| only sizes the allocation: a Mid minibatch reaches 66k of 1.08M possible vertices, and a
// table laid out for the bound (32 MB per minibatch, touched at random) pushed the feature rows out
// of the caches (the hit copy ran 20 % slower) besides missing L2 itself.  Which form a hop takes is
// decided per minibatch on the device, from the hop's size.
//
// Launches per call with fanouts: six per hop (two for each scan, the sample kernel, the
// deduplication) and the last hop's relabel; the seeds are put in place at the head of hop 1's first
// scan launch and the relabel of hop h-1 rides at the head of hop h's.  The per-minibatch pointers
// (a table too large for an argument block) stay on the device between calls and are stored again
// only when a call brings other buffers.
//
// The same machinery serves the sampler with given transition probabilities (Sec. 3.1, paragraph
// after Prop. 1): a target takes every entry of its row independently with the entry's probability,
// so step 1 is a counting pass with the random draws (one wavefront per target, ballots) and step 2
// repeats the draws to place the taken entries; no fanout bounds the sizes, so the counting pass
// also checks the caller's capacities and abandons a minibatch that would exceed them.
#include "spp_common.h"
#include "spp_device.h"

namespace spp {

constexpr int kMaxBatches = SPP_MAX_SAMPLE_BATCHES;

// What differs between the minibatches of one call (stored in device memory once per call).
struct BatchDesc {
    const int32_t* seeds;
    int32_t*       S;                   // node ids
    int32_t*       indptr[SPP_MAX_L];
    int32_t*       src[SPP_MAX_L];
    int64_t*       counts;              // n[0..MAX_L], e[0..MAX_L]
    uint32_t*      tinfo;               // [0] mask, [1] shift of the table for the current hop, [2] abandoned (workspace),
                                        // [3] log2 of the LDS partitions of the current hop, or kGlobalTable
    unsigned long long* taken;          // 64-bit count of taken entries of the current hop (given probabilities only)
    int64_t        ncap;                // capacities of the caller's buffers (checked on the device
    int64_t        ecap[SPP_MAX_L];     //   only when sizes are not bounded by fanouts)
    int32_t        nseeds;
    uint32_t       batch_lo;
};
struct BatchTable {
    BatchDesc b[kMaxBatches];
};
// What changes from call to call even when the caller reuses its buffers: the seeds and the number
// of the minibatch.  It rides in the argument block of the call's first launch, which stores it
// into the table; the rest of the table stays on the device between calls.
struct BatchDyn {
    const int32_t* seeds;
    int32_t        nseeds;
    uint32_t       batch_lo;
};
struct BatchDynAll {
    BatchDyn d[kMaxBatches];
};

// What the minibatches of one call share.
struct SampleArgs {
    const int64_t* rowptr;
    const int32_t* col;
    int64_t        N;
    unsigned long long* tab;            // one region of `cap` entries per minibatch
    int64_t        cap;                 // slots per region (a power of two, sized for the bound on |S_L|)
    int32_t*       flat;                // one region of `flat_stride` entries per minibatch, in flat (edge) order: what
                                        // every sampled id of the current hop resolved to (an index into S_{h-1}, or
                                        // n_{h-1} + the flat position of the id's first appearance); with the table in
                                        // global memory, until the scan's first pass, the table slot of the id
    int32_t*       gids;                // the same shape: the sampled ids themselves
    int64_t        flat_stride;
    int64_t*       row0;                // one region of `node_stride` entries per minibatch: where the row of the i-th
    int32_t*       deg;                 // vertex of S starts in col[], and its length (fanout sampling: read from rowptr
    int64_t        node_stride;         // once, when the vertex joins S; every later pass reads these in order)
    unsigned long long* totals;         // context-wide running sums: [0] batches, [1] |S_L|, [2] edges
    int*           bad;
    int*           bad_next;            // the next call's flags: cleared by this call's last kernel
    int            L;
    int            h;                   // hop, 1-based
    int            f;                   // fanout of this hop
    uint64_t       seed;
    const float*   t;                   // this hop's transition probabilities (aligned with col), or null: fanout sampling
    int32_t*       cnt;                 // one region of `cnt_stride` per-target counts per minibatch (given probabilities)
    int64_t        cnt_stride;
    int*           ovf;                 // set when a minibatch was abandoned for lack of capacity
    int            force_global;        // SPP_SAMPLE_GLOBAL_TABLE: every hop deduplicates in the global-memory table
};

__device__ __forceinline__ unsigned long long* tab_of(const SampleArgs& a, int j) { return a.tab + (int64_t)j * a.cap; }
__device__ __forceinline__ int32_t* flat_of(const SampleArgs& a, int j) { return a.flat + (int64_t)j * a.flat_stride; }
__device__ __forceinline__ int32_t* gids_of(const SampleArgs& a, int j) { return a.gids + (int64_t)j * a.flat_stride; }
__device__ __forceinline__ int64_t* row0_of(const SampleArgs& a, int j) { return a.row0 + (int64_t)j * a.node_stride; }
__device__ __forceinline__ int32_t* deg_of(const SampleArgs& a, int j) { return a.deg + (int64_t)j * a.node_stride; }
__device__ __forceinline__ int32_t* cnt_of(const SampleArgs& a, int j) { return a.cnt + (int64_t)j * a.cnt_stride; }
constexpr int kE = SPP_MAX_L + 1;      // offset of e[] inside counts

// Zeroes the counts of the new minibatches, stores what this call brings (seeds, minibatch number)
// into the table and copies the seeds into S_0.  x-th of gx workgroups of minibatch j.
__device__ __forceinline__ void seeds_rows(const SampleArgs& a, BatchTable* t, const BatchDyn& dyn, int j, unsigned x,
                                           unsigned gx) {
    BatchDesc& b = t->b[j];
    if (x == 0 && threadIdx.x == 0) {
        int64_t* c = b.counts;
        for (int k = 1; k <= SPP_MAX_L; ++k) c[k] = 0;
        for (int k = 0; k <= SPP_MAX_L; ++k) c[kE + k] = 0;
        c[0] = dyn.nseeds;
        b.seeds = dyn.seeds; b.nseeds = dyn.nseeds; b.batch_lo = dyn.batch_lo;
        b.tinfo[2] = 0;
        if (b.taken) *b.taken = 0ull;
    }
    for (int64_t i = (int64_t)x * kBlock + threadIdx.x; i < dyn.nseeds; i += (int64_t)gx * kBlock) {
        int32_t v = dyn.seeds[i];
        if (v < 0 || v >= a.N) { v = 0; atomicOr(a.bad, 1); }       // reported; keeps later row reads in range
        b.S[i] = v;
        if (!a.t && i < a.node_stride) {
            const int64_t r0 = a.rowptr[v];
            row0_of(a, j)[i] = r0;
            deg_of(a, j)[i] = (int32_t)(a.rowptr[v + 1] - r0);
        }
    }
}
__global__ void __launch_bounds__(kBlock) seeds_kernel(SampleArgs a, BatchTable* t, BatchDynAll dyn) {
    const BatchBlock bb = batch_block();
    seeds_rows(a, t, dyn.d[bb.j], bb.j, bb.x, gridDim.x);
}
// The same riding at the head of the first launch of hop 1's scan (fanout sampling), whose values
// then come from the seeds themselves: the table's copy is written by that very launch.
struct SeedsHead {
    SampleArgs a; BatchTable* t; BatchDynAll dyn;
    __device__ void operator()(int j, unsigned x, unsigned gx) const { seeds_rows(a, t, dyn.d[j], j, x, gx); }
};
struct CountInSeeds {
    SampleArgs a; BatchDynAll dyn;
    __device__ int64_t n(int j) const { return dyn.d[j].nseeds; }
    __device__ int operator()(int j, int64_t i) const {
        int32_t v = dyn.d[j].seeds[i];
        if (v < 0 || v >= a.N) v = 0;
        const int64_t d = a.rowptr[v + 1] - a.rowptr[v];
        return d < a.f ? (int)d : a.f;
    }
};

// ---- step 1 ----
// With given probabilities sizes are not bounded by fanouts: the 64-bit count of the counting pass
// decides whether the caller's buffers (and the table region laid out for them) hold this hop.
// The count stays as it is until the hop's last scan resets it, so every workgroup of a launch
// reads the same decision.
__device__ __forceinline__ bool hop_overflows(const SampleArgs& a, const BatchDesc& b) {
    return a.t != nullptr && *b.taken > (unsigned long long)b.ecap[a.h - 1];
}
// The flag tinfo[2] ("this minibatch was abandoned") is set by the Fin step of a scan, i.e. by one
// thread of a launch whose other workgroups read it.  Every reader in such a launch therefore ORs
// the flag with the condition under which that launch's Fin sets it, a condition that does not
// change during the launch (the hop's count of taken entries against the edge capacity in the
// offsets' scan; the scan's total against the vertex capacity in the scan that numbers the new
// vertices): whichever value of the flag a workgroup happens to see, the outcome is the same.
struct CountIn {
    SampleArgs a; const BatchTable* t;
    __device__ int64_t n(int j) const { return t->b[j].tinfo[2] || hop_overflows(a, t->b[j]) ? 0 : t->b[j].counts[a.h - 1]; }
    __device__ int64_t n(int j, int) const { return n(j); }
    __device__ int operator()(int j, int64_t i) const {
        if (a.t) return cnt_of(a, j)[i];
        const int d = deg_of(a, j)[i];
        return d < a.f ? d : a.f;
    }
};
struct CountOut {
    SampleArgs a; const BatchTable* t;
    __device__ void operator()(int j, int64_t i, int ex, int, int) const { t->b[j].indptr[a.h - 1][i] = ex; }
};
// This hop's table: the smallest power of two >= 2 (n_{h-1} + e_h), at least 1024 slots, never more
// than the region (the host sized it for the bound, which dominates).
__device__ __forceinline__ void hop_table(const SampleArgs& a, int64_t n_prev, int e_h, uint32_t& capj, int& shift) {
    const uint64_t want = 2ull * (uint64_t)(n_prev + (int64_t)(uint32_t)e_h);
    capj = 1024;
    shift = 22;
    while (capj < want && (int64_t)capj < a.cap) { capj <<= 1; --shift; }
}
// Where a hop's ids are deduplicated: in LDS, dealt to 2^k partitions of at most kLdsPartKeys ids on
// average (k returned), or in the table in global memory (kGlobalTable).  A function of the hop's size
// alone, so every workgroup of a launch that has the scan's total takes the same decision.
constexpr int kLdsSlots = 16384;                 // slots of a partition's table (64-bit entries: 128 KB of LDS)
constexpr int kLdsPartKeys = kLdsSlots / 2;
constexpr int kLdsMaxPartsLog2 = 4;
constexpr uint32_t kGlobalTable = 0xFFFFFFFFu;
__device__ __forceinline__ uint32_t hop_mode(const SampleArgs& a, int64_t n_prev, int e_h) {
    const int64_t keys = n_prev + (int64_t)(uint32_t)e_h;
    if (a.t != nullptr || a.force_global || keys > ((int64_t)kLdsPartKeys << kLdsMaxPartsLog2)) return kGlobalTable;
    uint32_t k = 0;
    while (((int64_t)kLdsPartKeys << k) < keys) ++k;
    return k;
}
struct CountFin {
    SampleArgs a; const BatchTable* t;
    __device__ void operator()(int j, int total) const {
        int64_t* c = t->b[j].counts;
        if (t->b[j].tinfo[2]) return;                        // abandoned at an earlier hop
        if (hop_overflows(a, t->b[j])) {
            t->b[j].tinfo[2] = 1;
            atomicOr(a.ovf, 1);
            return;
        }
        t->b[j].indptr[a.h - 1][c[a.h - 1]] = total;
        c[kE + a.h] = total;
        atomicAdd(&a.totals[2], (unsigned long long)(uint32_t)total);
        uint32_t capj;
        int shift;
        hop_table(a, c[a.h - 1], total, capj, shift);
        t->b[j].tinfo[0] = capj - 1;
        t->b[j].tinfo[1] = (uint32_t)shift;
        t->b[j].tinfo[3] = hop_mode(a, c[a.h - 1], total);
    }
};

// ---- step 2 ----
// Empties the part of the region that this hop's table occupies.  Rides at the end of the launch
// that writes the hop's offsets; the table's size follows from the scan's total, which every
// workgroup of that launch has.
struct TableClear {
    SampleArgs a; const BatchTable* t;
    __device__ void operator()(int j, unsigned x, unsigned gx, int total) const {
        if (t->b[j].tinfo[2] || hop_overflows(a, t->b[j])) return;
        if (hop_mode(a, t->b[j].counts[a.h - 1], total) != kGlobalTable) return;     // deduplicated in LDS: no table to empty
        unsigned long long* tab = tab_of(a, j);
        uint32_t capj;
        int shift;
        hop_table(a, t->b[j].counts[a.h - 1], total, capj, shift);
        const int64_t stride = (int64_t)gx * kBlock;
        for (int64_t i = (int64_t)x * kBlock + threadIdx.x; i < (int64_t)capj; i += stride) tab[i] = ~0ull;
    }
};

template <int G>
__global__ void __launch_bounds__(kBlock) sample_kernel(SampleArgs a, const BatchTable* __restrict__ t) {
    const BatchBlock bb = batch_block();
    const int jb = bb.j;
    const int lane = lane_id();
    const int j = lane & (G - 1);                  // slot handled by this lane
    const int gbase = lane - j;                    // first lane of the group inside the wavefront
    const uint64_t gmask = (G == 64) ? ~0ull : (((1ull << (G & 63)) - 1ull) << gbase);
    constexpr int kGroupsPerWave = kWave / G;
    const int64_t n_prev = t->b[jb].counts[a.h - 1];
    const uint32_t batch_lo = t->b[jb].batch_lo;
    const int64_t wave = ((int64_t)bb.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    const int f = a.f;
    const int32_t* __restrict__ S = t->b[jb].S;
    const int32_t* __restrict__ indptr = t->b[jb].indptr[a.h - 1];
    int32_t* __restrict__ flat = flat_of(a, jb);
    int32_t* __restrict__ gids = gids_of(a, jb);
    const int64_t* __restrict__ row0 = row0_of(a, jb);
    const int32_t* __restrict__ deg = deg_of(a, jb);
    unsigned long long* tab = tab_of(a, jb);
    const uint32_t mask = t->b[jb].tinfo[0];
    const int shift = (int)t->b[jb].tinfo[1];
    const bool global_table = t->b[jb].tinfo[3] == kGlobalTable;

    for (int64_t first = wave * kGroupsPerWave; first < n_prev; first += nwaves * kGroupsPerWave) {
        const int64_t i = first + (lane / G);
        const bool valid = i < n_prev;
        int64_t r0 = 0, d = 0;
        int32_t off = 0, v = 0;
        if (valid) {
            v = S[i];
            r0 = row0[i];
            d = deg[i];
            off = indptr[i];
        }
        const bool floyd = d > f;
        const int c = floyd ? f : (int)d;
        int64_t pos = j;                           // d <= f: the whole row, in row order
        if (floyd) {
            // Floyd's subset algorithm, one draw per slot: m = d - f + j, t uniform on [0, m]
            const uint64_t m = (uint64_t)(d - f + j);
            uint64_t tt = 0;
            if (j < f) {
                const uint32_t r = rand32(a.seed, batch_lo, (uint32_t)a.h, (uint32_t)v, (uint32_t)j);
                tt = ((uint64_t)r * (m + 1ull)) >> 32;
            }
            pos = (int64_t)tt;
            // slot jj takes t_jj unless an earlier slot already holds it, else m_jj (never held before)
            for (int jj = 1; jj < f; ++jj) {
                const int64_t tj = __shfl((long long)tt, gbase + jj, kWave);
                const bool hit = (j < jj) && (pos == tj);
                const uint64_t b = __ballot(hit) & gmask;
                if (j == jj && b != 0ull) pos = (int64_t)m;
            }
        }
        const bool mine = valid && j < c;
        int32_t gid = 0;
        int64_t e = -1;                            // flat position of this lane's sampled id, if it has one
        if (mine) {
            gid = a.col[r0 + pos];
            e = (int64_t)off + j;
            gids[e] = gid;
        }
        if (!global_table) continue;               // the ids meet in LDS, in the launch that follows
        // the table was emptied for this hop, so the target is offered again with its index; the
        // group's last lane does it when it has no neighbour of its own (c < G), else lane 0 after
        // its neighbour
        const bool spare = c < G;
        uint32_t key = 0, val = 0;
        bool ins = false;
        if (mine) {
            key = (uint32_t)gid; val = (uint32_t)(n_prev + e); ins = true;
        } else if (valid && spare && j == G - 1) {
            key = (uint32_t)v; val = (uint32_t)i; ins = true;
        }
        if (ins) {
            const uint32_t slot = table_insert_min(tab, mask, shift, key, val);
            if (e >= 0) flat[e] = (int32_t)slot;
        }
        if (valid && !spare && j == 0) table_insert_min(tab, mask, shift, (uint32_t)v, (uint32_t)i);
    }
}

// ---- step 3 in LDS ----
// One workgroup per (partition, minibatch).  An id belongs to the partition named by the top bits of
// its hash; its slot comes from the bits below.  Entries are (id << 32 | position), empty = all ones;
// an insertion keeps the smallest position offered for an id.  A partition holds 8192 ids on average
// and 16384 at most; more than that in one partition (ids that share their hash's top bits by the
// thousand) cannot be held: the call then reports an error and the minibatch's output is not valid.
constexpr int kDedupBlock = 1024;
__device__ __forceinline__ bool lds_insert_min(unsigned long long* tab, uint32_t slot, uint32_t key, uint32_t value) {
    const unsigned long long want = ((unsigned long long)key << 32) | value;
    for (int probes = 0; probes < kLdsSlots; ++probes) {
        unsigned long long cur = tab[slot];
        if (cur == kEmpty) {
            const unsigned long long old = atomicCAS(&tab[slot], (unsigned long long)kEmpty, want);
            if (old == kEmpty) return true;
            cur = old;
        }
        if ((uint32_t)(cur >> 32) == key) {
            if (want < cur) atomicMin(&tab[slot], want);
            return true;
        }
        slot = (slot + 1) & (kLdsSlots - 1);
    }
    return false;
}
__device__ __forceinline__ uint32_t lds_find(const unsigned long long* tab, uint32_t slot, uint32_t key) {
    for (int probes = 0; probes < kLdsSlots; ++probes) {
        const unsigned long long cur = tab[slot];
        if ((uint32_t)(cur >> 32) == key) return (uint32_t)cur;
        if (cur == kEmpty) break;
        slot = (slot + 1) & (kLdsSlots - 1);
    }
    return 0xFFFFFFFFu;                            // not reached for an id that was inserted
}
// Only one id in 2^k belongs to the workgroup's partition, so the ids that do are first gathered, per
// wavefront, in a small queue in LDS (ballot, rank among the lanes that have one) and handed out 64
// at a time: the atomics of an insertion then run with every lane busy.  (With each lane inserting
// the ids it had read itself, an atomic instruction served 8 lanes of 64 and the LDS pipeline, which
// takes one instruction at a time, set the pace: 0.37 ms for the last hop of 64 minibatches.)
constexpr int kQueue = 2 * kWave;                 // entries a wavefront's queue holds
struct WaveQueue {
    unsigned long long* q;                        // this wavefront's kQueue entries: (id << 32 | payload)
    int n;                                        // entries queued (the same in every lane)
    // Queues `item` of the lanes where `has` is set.  Returns true when 64 entries are ready: `out` is
    // this lane's (the queue keeps the rest).
    __device__ __forceinline__ bool push(bool has, unsigned long long item, unsigned long long& out) {
        const uint64_t m = __ballot(has);
        if (has) q[n + __popcll(m & ((1ull << lane_id()) - 1ull))] = item;
        n += __popcll(m);
        if (n < kWave) return false;
        out = q[lane_id()];
        const unsigned long long rest = q[kWave + lane_id()];     // n < 2 * 64: at most 64 entries stay
        n -= kWave;
        if (lane_id() < n) q[lane_id()] = rest;
        return true;
    }
    // What is left at the end: true in the lanes that get an entry.
    __device__ __forceinline__ bool drain(unsigned long long& out) {
        const bool mine = lane_id() < n;
        if (mine) out = q[lane_id()];
        n = 0;
        return mine;
    }
};

__global__ void __launch_bounds__(kDedupBlock) dedup_lds_kernel(SampleArgs a, const BatchTable* __restrict__ t) {
    extern __shared__ unsigned long long ltab[];
    const int jb = blockIdx.x;                     // partitions are the slow index: the workgroups of partitions
    const uint32_t part = blockIdx.y;              // that a minibatch does not use come last and leave at once
    const uint32_t k = t->b[jb].tinfo[3];
    if (t->b[jb].tinfo[2] || k == kGlobalTable || part >= (1u << k)) return;
    const int64_t n_prev = t->b[jb].counts[a.h - 1];
    const int64_t e_h = t->b[jb].counts[kE + a.h];
    const int32_t* __restrict__ S = t->b[jb].S;
    const int32_t* __restrict__ gids = gids_of(a, jb);
    int32_t* __restrict__ flat = flat_of(a, jb);
    WaveQueue wq;
    wq.q = ltab + kLdsSlots + (threadIdx.x >> 6) * kQueue;
    wq.n = 0;
    for (int i = threadIdx.x; i < kLdsSlots; i += kDedupBlock) ltab[i] = kEmpty;
    __syncthreads();
    // hash bits: the top k name the partition, the 14 below them the slot
    auto mine = [&](uint32_t key) { return k == 0 || ((key * 0x9E3779B1u) >> (32 - k)) == part; };
    auto slot_of = [&](uint32_t key) { return ((key * 0x9E3779B1u) << k) >> (32 - 14); };
    // The lists are short (tens of thousands of ids) and every workgroup of the minibatch reads all of
    // them, so a pass is a chain of L2 round trips: eight loads per thread are in flight at a time.
    // Whole wavefronts walk the rounds together (the queue's ballots need every lane).
    constexpr int kU = 8;
    bool ok = true;
    auto insert = [&](unsigned long long item) {
        const uint32_t key = (uint32_t)(item >> 32);
        ok = lds_insert_min(ltab, slot_of(key), key, (uint32_t)item) && ok;
    };
    auto insert_all = [&](const int32_t* __restrict__ ids, int64_t count, int64_t first_value) {
        const int64_t rounds = (count + (int64_t)kDedupBlock * kU - 1) / ((int64_t)kDedupBlock * kU);
        for (int64_t r = 0; r < rounds; ++r) {
            const int64_t i0 = r * kDedupBlock * kU + threadIdx.x;
            uint32_t key[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u)
                if (i0 + u * kDedupBlock < count) key[u] = (uint32_t)ids[i0 + u * kDedupBlock];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const bool has = i0 + u * kDedupBlock < count && mine(key[u]);
                unsigned long long item;
                if (wq.push(has, ((unsigned long long)key[u] << 32) | (uint32_t)(first_value + i0 + u * kDedupBlock), item)) insert(item);
            }
        }
    };
    insert_all(S, n_prev, 0);
    insert_all(gids, e_h, n_prev);
    {
        unsigned long long item;
        if (wq.drain(item)) insert(item);
    }
    if (!ok) atomicOr(a.bad, 4);
    __syncthreads();
    auto resolve = [&](unsigned long long item) {
        const uint32_t key = (uint32_t)(item >> 32);
        flat[(uint32_t)item] = (int32_t)lds_find(ltab, slot_of(key), key);
    };
    const int64_t rounds = (e_h + (int64_t)kDedupBlock * kU - 1) / ((int64_t)kDedupBlock * kU);
    for (int64_t r = 0; r < rounds; ++r) {
        const int64_t e0 = r * kDedupBlock * kU + threadIdx.x;
        uint32_t key[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u)
            if (e0 + u * kDedupBlock < e_h) key[u] = (uint32_t)gids[e0 + u * kDedupBlock];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const bool has = e0 + u * kDedupBlock < e_h && mine(key[u]);
            unsigned long long item;
            if (wq.push(has, ((unsigned long long)key[u] << 32) | (uint32_t)(e0 + u * kDedupBlock), item)) resolve(item);
        }
    }
    {
        unsigned long long item;
        if (wq.drain(item)) resolve(item);
    }
}

// ---- steps 1 and 2 with given transition probabilities ----
// Entry k of v's row is taken iff rand32(seed, batch, hop, v, k) < floor(t * 2^32); a probability
// outside [0, 1] counts as 0 and is reported.  A lane decides four consecutive entries at a time:
// their draws are the four words of one Philox block (that is how rand32 numbers them).
// Returns the 4-bit mask of the taken ones among entries k4 .. k4+3 (k4 a multiple of 4) of a row of d.
__device__ __forceinline__ uint32_t general_take4(const SampleArgs& a, uint32_t batch_lo, int64_t v, int64_t r0, int64_t k4,
                                                  int64_t d) {
    if (k4 >= d) return 0u;
    const Philox4 p = philox4x32_10((uint32_t)v, (uint32_t)(k4 >> 2), (uint32_t)a.h, batch_lo, (uint32_t)a.seed,
                                    (uint32_t)(a.seed >> 32));
    uint32_t m = 0u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (k4 + i < d) {
            const float tt = a.t[r0 + k4 + i];
            if (!(tt >= 0.0f && tt <= 1.0f)) { atomicOr(a.bad, 2); continue; }
            const uint64_t thr = (uint64_t)((double)tt * 4294967296.0);
            if ((uint64_t)p.w[i] < thr) m |= 1u << i;
        }
    }
    return m;
}
// A row is walked by a group of G lanes (G = 16: four targets per wavefront; G = 64: one), 4 G
// entries per step.  Most rows hold a handful of entries, a few tens of thousands: rows of at most
// kShortRow entries are taken four per wavefront in a first sweep over the targets, longer ones by
// a whole wavefront in a second sweep.
constexpr int kShortRow = 256;
constexpr int kShortGroup = 16;

// Taken entries among the 4 G entries a group decides in one step: in all of the group's lanes, and
// in its lanes below this one.  gmask = the group's lanes, lt_mask = the wavefront's lanes below this one.
__device__ __forceinline__ int taken_in_group(uint32_t m, uint64_t gmask, uint64_t lt_mask, int& below) {
    int all = 0;
    below = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint64_t b = __ballot((m >> i) & 1u) & gmask;
        all += __popcll(b);
        below += __popcll(b & lt_mask);
    }
    return all;
}

// Which target a lane group works on in sweep `longer` (0: short rows, G = kShortGroup; 1: long rows, G = 64).
struct GroupWalk {
    int64_t first, stride;      // first target of this group and the step to its next one
    uint32_t glane;             // lane inside the group
    uint64_t gmask;             // the group's lanes
};
template <int G>
__device__ __forceinline__ GroupWalk group_walk(const BatchBlock& bb) {
    const int lane = lane_id();
    const int64_t wave = ((int64_t)bb.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    GroupWalk w;
    w.first = wave * (kWave / G) + lane / G;
    w.stride = nwaves * (kWave / G);
    w.glane = (uint32_t)(lane % G);
    w.gmask = G == kWave ? ~0ull : ((1ull << (G & 63)) - 1ull) << (lane - lane % G);
    return w;
}

template <int G>
__device__ __forceinline__ void general_count_rows(const SampleArgs& a, const BatchDesc& b, const BatchBlock& bb,
                                                   int32_t* __restrict__ cnt, unsigned long long& mine) {
    const GroupWalk w = group_walk<G>(bb);
    const int64_t n_prev = b.counts[a.h - 1];
    const int64_t rounds = (n_prev + w.stride - 1) / w.stride;           // whole wavefronts reach the ballots
    for (int64_t it = 0; it < rounds; ++it) {
        const int64_t i = w.first + it * w.stride;
        int64_t v = 0, r0 = 0, d = 0;
        if (i < n_prev) {
            v = b.S[i];
            r0 = a.rowptr[v];
            d = a.rowptr[v + 1] - r0;
            if ((d > kShortRow) != (G == kWave)) d = 0;                  // the other sweep's row
        }
        int64_t c = 0;
        // groups of one wavefront walk rows of different lengths: all step until the longest is done
        for (int64_t k0 = 0; __any(k0 < d); k0 += 4 * G) {
            int below;
            c += taken_in_group(k0 < d ? general_take4(a, b.batch_lo, v, r0, k0 + 4 * w.glane, d) : 0u, w.gmask, 0ull, below);
        }
        // a count beyond any capacity is stored saturated; the 64-bit total decides
        if (i < n_prev && w.glane == 0 && ((a.rowptr[v + 1] - a.rowptr[v] > kShortRow) == (G == kWave))) {
            cnt[i] = (int32_t)(c < 0x7FFFFFFFll ? c : 0x7FFFFFFFll);
            mine += (unsigned long long)c;
        }
    }
}

__global__ void __launch_bounds__(kBlock) general_count_kernel(SampleArgs a, const BatchTable* __restrict__ t) {
    __shared__ unsigned long long red[kBlock];
    const BatchBlock bb = batch_block();
    const int jb = bb.j;
    if (t->b[jb].tinfo[2]) return;
    unsigned long long mine = 0;
    general_count_rows<kShortGroup>(a, t->b[jb], bb, cnt_of(a, jb), mine);
    general_count_rows<kWave>(a, t->b[jb], bb, cnt_of(a, jb), mine);
    red[threadIdx.x] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long s = 0;
        for (int k = 0; k < kBlock; ++k) s += red[k];
        if (s) atomicAdd(t->b[jb].taken, s);
    }
}

template <int G>
__device__ __forceinline__ void general_sample_rows(const SampleArgs& a, const BatchDesc& b, const BatchBlock& bb,
                                                    int32_t* __restrict__ flat, int32_t* __restrict__ gids,
                                                    unsigned long long* tab) {
    const GroupWalk w = group_walk<G>(bb);
    const int lane = lane_id();
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    const int64_t n_prev = b.counts[a.h - 1];
    const int32_t* __restrict__ indptr = b.indptr[a.h - 1];
    const uint32_t mask = b.tinfo[0];
    const int shift = (int)b.tinfo[1];
    const int64_t rounds = (n_prev + w.stride - 1) / w.stride;
    for (int64_t it = 0; it < rounds; ++it) {
        const int64_t i = w.first + it * w.stride;
        int64_t v = 0, r0 = 0, d = 0, e = 0;
        if (i < n_prev) {
            v = b.S[i];
            r0 = a.rowptr[v];
            d = a.rowptr[v + 1] - r0;
            if ((d > kShortRow) != (G == kWave)) d = 0;
            else {
                e = indptr[i];
                // the table was emptied for this hop, so the target is offered again with its index
                if (w.glane == 0) table_insert_min(tab, mask, shift, (uint32_t)v, (uint32_t)i);
            }
        }
        for (int64_t k0 = 0; __any(k0 < d); k0 += 4 * G) {
            const int64_t k4 = k0 + 4 * w.glane;
            const uint32_t m = k0 < d ? general_take4(a, b.batch_lo, v, r0, k4, d) : 0u;
            int below;
            const int all = taken_in_group(m, w.gmask, lt_mask, below);
            int64_t pos = e + below;                   // entries ascend with the lane, then inside the lane
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if ((m >> q) & 1u) {
                    const int32_t gid = a.col[r0 + k4 + q];
                    gids[pos] = gid;
                    flat[pos] = (int32_t)table_insert_min(tab, mask, shift, (uint32_t)gid, (uint32_t)(n_prev + pos));
                    ++pos;
                }
            }
            e += all;
        }
    }
}

__global__ void __launch_bounds__(kBlock) general_sample_kernel(SampleArgs a, const BatchTable* __restrict__ t) {
    const BatchBlock bb = batch_block();
    const int jb = bb.j;
    if (t->b[jb].tinfo[2]) return;
    general_sample_rows<kShortGroup>(a, t->b[jb], bb, flat_of(a, jb), gids_of(a, jb), tab_of(a, jb));
    general_sample_rows<kWave>(a, t->b[jb], bb, flat_of(a, jb), gids_of(a, jb), tab_of(a, jb));
}

// ---- step 4 ----
struct NewIn {
    SampleArgs a; const BatchTable* t;
    __device__ int64_t n(int j) const { return t->b[j].tinfo[2] ? 0 : t->b[j].counts[kE + a.h]; }
    // With the table in global memory, what the entry resolved to is read from its slot here (a
    // random 8-byte read that moves a whole line) and kept in the slot's place; the outcome is left
    // in the entry's place in the hop's src array (-2 first appearance, -1 repeat) for the second pass.
    __device__ int operator()(int j, int64_t e) const {
        int32_t* __restrict__ flat = flat_of(a, j);
        uint32_t val = (uint32_t)flat[e];
        if (t->b[j].tinfo[3] == kGlobalTable) {
            val = (uint32_t)tab_of(a, j)[val];
            flat[e] = (int32_t)val;
        }
        const int first = (int64_t)val == t->b[j].counts[a.h - 1] + e ? 1 : 0;
        t->b[j].src[a.h - 1][e] = first ? -2 : -1;
        return first;
    }
};
// Whether the scan's total of new vertices exceeds the caller's vertex capacity (given probabilities only).
__device__ __forceinline__ bool ids_overflow(const SampleArgs& a, const BatchDesc& b, int total) {
    return a.t != nullptr && b.counts[a.h - 1] + (int64_t)(uint32_t)total > b.ncap;
}
struct NewInKept {
    SampleArgs a; const BatchTable* t;
    // second launch of the scan: NewFin of this launch abandons the minibatch exactly when ids_overflow()
    __device__ int64_t n(int j, int total) const {
        return t->b[j].tinfo[2] || ids_overflow(a, t->b[j], total) ? 0 : t->b[j].counts[kE + a.h];
    }
    __device__ int operator()(int j, int64_t e) const { return t->b[j].src[a.h - 1][e] == -2 ? 1 : 0; }
};
struct NewOut {
    SampleArgs a; const BatchTable* t;
    __device__ void operator()(int j, int64_t e, int ex, int v, int total) const {
        if (!v || t->b[j].tinfo[2] || ids_overflow(a, t->b[j], total)) return;    // NewFin abandons the minibatch
        // A first appearance gets its local id here; the relabel pass fills in the repeats.
        const int64_t n_prev = t->b[j].counts[a.h - 1];
        const int64_t id = n_prev + ex;
        const int32_t gid = gids_of(a, j)[e];
        t->b[j].src[a.h - 1][e] = (int32_t)id;
        t->b[j].S[id] = gid;
        // a vertex that will be a target of the next hop: its row is looked up here, once
        if (!a.t && a.h < a.L && id < a.node_stride) {
            const int64_t r0 = a.rowptr[gid];
            row0_of(a, j)[id] = r0;
            deg_of(a, j)[id] = (int32_t)(a.rowptr[gid + 1] - r0);
        }
    }
};
struct NewFin {
    SampleArgs a; const BatchTable* t;
    __device__ void operator()(int j, int total) const {
        int64_t* c = t->b[j].counts;
        if (a.t) *t->b[j].taken = 0ull;                    // the next hop counts from zero
        if (t->b[j].tinfo[2]) return;
        const int64_t n = c[a.h - 1] + (int64_t)(uint32_t)total;
        if (ids_overflow(a, t->b[j], total)) {             // the new ids do not fit the caller's buffer
            t->b[j].tinfo[2] = 1;
            atomicOr(a.ovf, 1);
            c[kE + a.h] = 0;
            return;
        }
        c[a.h] = n;
        if (a.h == a.L) { atomicAdd(&a.totals[1], (unsigned long long)n); atomicAdd(&a.totals[0], 1ull); }
    }
};

// ---- step 5 ----
// A repeated id takes the index of the earlier vertex it resolved to, or the local id that the scan
// gave to its first appearance (an entry before it in the same list, final since the launch before).
__device__ __forceinline__ void relabel_rows(const SampleArgs& a, const BatchTable* __restrict__ t, int j, unsigned x,
                                             unsigned gx) {
    if (t->b[j].tinfo[2]) return;
    const int64_t e_h = t->b[j].counts[kE + a.h];
    const int64_t n_prev = t->b[j].counts[a.h - 1];
    const int32_t* __restrict__ flat = flat_of(a, j);
    int32_t* src = t->b[j].src[a.h - 1];
    const int64_t stride = (int64_t)gx * kBlock;
    for (int64_t e = (int64_t)x * kBlock + threadIdx.x; e < e_h; e += stride)
        if (src[e] < 0) {
            const int64_t fp = (uint32_t)flat[e];
            src[e] = fp < n_prev ? (int32_t)fp : src[fp - n_prev];
        }
}
__global__ void __launch_bounds__(kBlock) relabel_kernel(SampleArgs a, const BatchTable* __restrict__ t) {
    const BatchBlock bb = batch_block();
    relabel_rows(a, t, bb.j, bb.x, gridDim.x);
    // the call's last launch: nothing of this call touches the other set of flags
    if (a.h == a.L && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 2) a.bad_next[threadIdx.x] = 0;
}
// The relabel of hop h-1 riding at the head of hop h's first scan launch (it reads the table, the
// flat ids and the counts of hop h-1, which that launch only reads too).
struct RelabelPrev {
    SampleArgs a; const BatchTable* t;         // a.h = the hop to relabel
    __device__ void operator()(int j, unsigned x, unsigned gx) const { relabel_rows(a, t, j, x, gx); }
};

// Stores a table of per-minibatch pointers in device memory, sixteen entries per launch (a launch's
// argument block holds 4 KB).  Only needed when a call brings buffers that no slot holds.
constexpr int kStoreChunk = 16;
struct BatchTableChunk { BatchDesc b[kStoreChunk]; };
__global__ void __launch_bounds__(kBlock) batch_table_store_kernel(BatchTableChunk src, BatchTable* dst, int first) {
    const uint64_t* s = reinterpret_cast<const uint64_t*>(&src);
    uint64_t* d = reinterpret_cast<uint64_t*>(&dst->b[first]);
    for (unsigned i = threadIdx.x; i < sizeof(BatchTableChunk) / sizeof(uint64_t); i += kBlock) d[i] = s[i];
}
// [0] error flag, [1] capacity flag of a call
__global__ void sample_flags_clear_kernel(int* bad) {
    if (threadIdx.x < 2) bad[threadIdx.x] = 0;
}
static_assert(sizeof(BatchTableChunk) % sizeof(uint64_t) == 0, "copied as 64-bit words");
static_assert(sizeof(BatchTableChunk) <= 4000, "must fit a launch's argument block");
static_assert(kMaxBatches % kStoreChunk == 0, "the table is stored in whole chunks");

}  // namespace spp

extern "C" int spp_mfg_bound(int32_t nseeds, const int32_t* fanouts, int32_t L, int64_t N,
                             int64_t* n_bound, int64_t* e_bound) {
    SPP_CHECK(fanouts && n_bound && e_bound, SPP_E_ARG, "spp_mfg_bound: null argument");
    SPP_CHECK(L >= 1 && L <= SPP_MAX_L && nseeds >= 0 && N > 0, SPP_E_ARG, "spp_mfg_bound: L = %d, nseeds = %d", L, nseeds);
    n_bound[0] = nseeds < N ? nseeds : N;
    e_bound[0] = 0;
    for (int h = 1; h <= L; ++h) {
        const int64_t f = fanouts[h - 1];
        SPP_CHECK(f >= 1 && f <= SPP_MAX_FANOUT, SPP_E_ARG, "spp_mfg_bound: fanout %lld of hop %d not in [1, %d]",
                  (long long)f, h, SPP_MAX_FANOUT);
        e_bound[h] = n_bound[h - 1] * f;
        const int64_t n = n_bound[h - 1] + e_bound[h];
        n_bound[h] = n < N ? n : N;
    }
    return SPP_OK;
}

// Both samplers: sizes bounded by `fanouts`, or (d_t given) every entry of a row taken with its
// own probability and sizes checked against the caller's capacities on the device.
static int sample_batches(spp_ctx* ctx, const spp_graph* g, const spp_sample_item* items, int32_t n_items,
                          const int32_t* fanouts, const float* const* d_t, int32_t L, uint64_t seed, uint32_t flags) {
    using namespace spp;
    const bool general = d_t != nullptr;
    SPP_CHECK(ctx && g && (fanouts || general) && (items || n_items == 0), SPP_E_ARG, "spp_sample_mfg: null argument");
    SPP_CHECK(n_items >= 0 && n_items <= SPP_MAX_SAMPLE_BATCHES, SPP_E_ARG, "spp_sample_mfg: %d minibatches (at most %d)",
              n_items, SPP_MAX_SAMPLE_BATCHES);
    SPP_CHECK(L >= 1 && L <= SPP_MAX_L, SPP_E_ARG, "spp_sample_mfg: L = %d not in [1, %d]", L, SPP_MAX_L);
    if (general)
        for (int h = 0; h < L; ++h)
            SPP_CHECK(d_t[h] || g->M == 0, SPP_E_ARG, "spp_sample_mfg_general: no transition probabilities for hop %d", h + 1);
    if (n_items == 0) return SPP_OK;
    BatchTable ht = {};             // what stays the same while the caller reuses its buffers
    BatchDynAll dyn = {};           // what every call brings
    int64_t nb[SPP_MAX_L + 1] = {0}, eb[SPP_MAX_L + 1] = {0};       // bounds (capacities) of the largest minibatch
    int max_seeds = 0;
    for (int j = 0; j < n_items; ++j) {
        const spp_sample_item& it = items[j];
        spp_mfg* io = it.io;
        SPP_CHECK(io, SPP_E_ARG, "spp_sample_mfg: minibatch %d has no output struct", j);
        SPP_CHECK(it.nseeds >= 0 && (it.d_seeds || it.nseeds == 0), SPP_E_ARG, "spp_sample_mfg: seeds of minibatch %d", j);
        SPP_CHECK(it.nseeds <= g->N, SPP_E_ARG, "spp_sample_mfg: more seeds than vertices");
        SPP_CHECK(io->d_node_ids && io->d_counts, SPP_E_ARG, "spp_sample_mfg: null output buffer");
        int64_t nbj[SPP_MAX_L + 1], ebj[SPP_MAX_L + 1];
        if (general) {
            // no fanout bounds the sizes: the capacities are the bounds, enforced on the device
            SPP_CHECK(io->n_nodes_cap >= it.nseeds && io->n_nodes_cap >= 1, SPP_E_CAPACITY,
                      "spp_sample_mfg_general: d_node_ids holds %lld entries, the minibatch has %d seeds",
                      (long long)io->n_nodes_cap, it.nseeds);
            ebj[0] = 0;
            for (int h = 0; h <= L; ++h) nbj[h] = io->n_nodes_cap;
            for (int h = 1; h <= L; ++h) {
                SPP_CHECK(io->n_edges_cap[h - 1] >= 0, SPP_E_ARG, "spp_sample_mfg_general: negative capacity of hop %d", h);
                ebj[h] = io->n_edges_cap[h - 1];
            }
        } else {
            SPP_TRY(spp_mfg_bound(it.nseeds, fanouts, L, g->N, nbj, ebj));
            SPP_CHECK(io->n_nodes_cap >= nbj[L] && io->n_nodes_cap >= 1, SPP_E_CAPACITY,
                      "spp_sample_mfg: d_node_ids holds %lld entries, the bound is %lld", (long long)io->n_nodes_cap, (long long)nbj[L]);
        }
        ht.b[j].ncap = io->n_nodes_cap;
        for (int h = 1; h <= L; ++h) {
            SPP_CHECK(io->d_indptr[h - 1] && io->d_src[h - 1], SPP_E_ARG, "spp_sample_mfg: null buffer of hop %d", h);
            SPP_CHECK(io->n_edges_cap[h - 1] >= ebj[h], SPP_E_CAPACITY,
                      "spp_sample_mfg: d_src of hop %d holds %lld entries, the bound is %lld", h,
                      (long long)io->n_edges_cap[h - 1], (long long)ebj[h]);
            SPP_CHECK(ebj[h] < 0x3FFFFFFFll && nbj[h] + ebj[h] < 0x3FFFFFFFll, SPP_E_ARG, "spp_sample_mfg: hop %d exceeds 30-bit sizes", h);
            ht.b[j].indptr[h - 1] = io->d_indptr[h - 1];
            ht.b[j].src[h - 1] = io->d_src[h - 1];
            ht.b[j].ecap[h - 1] = io->n_edges_cap[h - 1];
        }
        for (int h = 0; h <= L; ++h) { if (nbj[h] > nb[h]) nb[h] = nbj[h]; if (ebj[h] > eb[h]) eb[h] = ebj[h]; }
        dyn.d[j].seeds = it.d_seeds; dyn.d[j].nseeds = it.nseeds; dyn.d[j].batch_lo = (uint32_t)it.batch_index;
        ht.b[j].S = io->d_node_ids; ht.b[j].counts = io->d_counts;
        if (it.nseeds > max_seeds) max_seeds = it.nseeds;
    }
    int64_t emax = 1;
    for (int h = 1; h <= L; ++h) if (eb[h] > emax) emax = eb[h];
    SPP_HIP(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;

    // table region per minibatch: twice the most keys a hop can hold (all ids so far plus the hop's entries)
    const int64_t max_keys = general ? nb[L] + emax : nb[L];
    const uint32_t cap = next_pow2((uint64_t)(2 * max_keys > 1024 ? 2 * max_keys : 1024));
    // workgroups per minibatch in the scans and the table clear: the whole call gets about 4 per CU
    const int per_batch = (ctx->num_cu * 4 + n_items - 1) / n_items;
    const int scan_grid = ((per_batch < 32 ? 32 : per_batch) + 7) & ~7;     // multiples of 8: see batch_block()
    SPP_TRY(ctx->table.reserve((size_t)cap * sizeof(uint64_t) * n_items));
    SPP_TRY(ctx->flat.reserve((size_t)emax * sizeof(int32_t) * n_items * 2));        // what the ids resolve to, and the ids
    SPP_TRY(ctx->slots.reserve((size_t)(4 * sizeof(uint32_t) + sizeof(unsigned long long)) * kMaxBatches + 64 +
                               (general ? (size_t)nb[L] * sizeof(int32_t) * n_items : 0)));
    unsigned long long* taken = ctx->slots.as<unsigned long long>();
    uint32_t* tinfo = reinterpret_cast<uint32_t*>(taken + kMaxBatches);
    for (int j = 0; j < n_items; ++j) {
        ht.b[j].tinfo = tinfo + 4 * j;
        ht.b[j].taken = general ? taken + j : nullptr;
    }
    SPP_TRY(ctx->partials.reserve((size_t)scan_grid * n_items * sizeof(int) + 64));
    int* partial = ctx->partials.as<int>();
    // The table of per-minibatch pointers is too large to ride in the argument block of every kernel, so it
    // lives in device memory: in one of a few slots, found again by content when a later call brings the same
    // buffers (then nothing is stored), else stored over the slot used longest ago.
    constexpr int kSlots = spp_ctx::kBatchSlots;
    if (!ctx->btab.ptr) {
        SPP_TRY(ctx->btab.reserve(kSlots * sizeof(BatchTable) + 256));
        for (int k = 0; k < kSlots; ++k) ctx->btab_n[k] = 0;
        ctx->sample_flags_clean = 0;
    }
    if (!ctx->btab_mirror) {
        ctx->btab_mirror = calloc(kSlots, sizeof(BatchTable));
        SPP_CHECK(ctx->btab_mirror, SPP_E_OOM, "spp_sample_mfg: out of host memory");
    }
    BatchTable* mirror = static_cast<BatchTable*>(ctx->btab_mirror);
    int slot = -1;
    for (int k = 0; k < kSlots && slot < 0; ++k)
        if (ctx->btab_n[k] == n_items && memcmp(&mirror[k], &ht, (size_t)n_items * sizeof(BatchDesc)) == 0) slot = k;
    const bool stored = slot >= 0;
    if (!stored) {
        slot = 0;
        for (int k = 1; k < kSlots; ++k)
            if (ctx->btab_stamp[k] < ctx->btab_stamp[slot]) slot = k;
        ctx->btab_n[slot] = 0;          // until its launches are enqueued
    }
    ctx->btab_stamp[slot] = ++ctx->sample_calls;
    BatchTable* dt = ctx->btab.as<BatchTable>() + slot;
    // two sets of flags, used alternately: this call's were cleared by the last kernel of the call before
    int* flags2 = reinterpret_cast<int*>(ctx->btab.as<BatchTable>() + kSlots);
    int* d_bad = flags2 + 2 * (ctx->sample_calls & 1);
    int* d_bad_next = flags2 + 2 * ((ctx->sample_calls + 1) & 1);
    const bool flags_clean = ctx->sample_flags_clean != 0;
    ctx->sample_flags_clean = 0;        // set again once this call's last kernel is enqueued

    SampleArgs a;
    a.rowptr = g->rowptr; a.col = g->col; a.N = g->N;
    a.tab = ctx->table.as<unsigned long long>(); a.cap = cap;
    a.flat = ctx->flat.as<int32_t>(); a.flat_stride = emax;
    a.gids = a.flat + (size_t)emax * n_items;
    // row start and length of every vertex that can be a target: the members of S_{L-1}
    a.node_stride = general ? 0 : nb[L - 1];
    SPP_TRY(ctx->nodeinfo.reserve((size_t)a.node_stride * n_items * (sizeof(int64_t) + sizeof(int32_t)) + 64));
    a.row0 = ctx->nodeinfo.as<int64_t>();
    a.deg = reinterpret_cast<int32_t*>(a.row0 + (size_t)a.node_stride * n_items);
    const size_t dedup_lds = ((size_t)kLdsSlots + (size_t)(kDedupBlock / kWave) * kQueue) * sizeof(unsigned long long);
    if (!general && !ctx->dedup_lds_set) {
        SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&dedup_lds_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)dedup_lds));
        ctx->dedup_lds_set = 1;
    }
    a.totals = reinterpret_cast<unsigned long long*>(ctx->totals); a.bad = d_bad; a.ovf = d_bad + 1; a.bad_next = d_bad_next;
    a.L = L; a.h = 0; a.f = 0; a.seed = seed;
    a.t = nullptr;
    a.force_global = (flags & SPP_SAMPLE_GLOBAL_TABLE) ? 1 : 0;
    a.cnt = reinterpret_cast<int32_t*>(tinfo + 4 * kMaxBatches + 16); a.cnt_stride = nb[L];

    auto capped = [&](int64_t need, int64_t lim) {
        const int64_t g = need < 1 ? 1 : (need < lim ? need : lim);
        return (unsigned)((g + 7) & ~(int64_t)7);
    };
    const int64_t share = (int64_t)ctx->num_cu * 64 / n_items + 1;    // workgroups per minibatch in the wide kernels
    {
        ScopedTimer tt(ctx, SPP_T_SAMPLE, st);
        if (!flags_clean) sample_flags_clear_kernel<<<1, 64, 0, st>>>(d_bad);
        if (!stored) {
            for (int first = 0; first < n_items; first += kStoreChunk) {
                BatchTableChunk chunk;
                memcpy(&chunk, &ht.b[first], sizeof(chunk));
                batch_table_store_kernel<<<1, kBlock, 0, st>>>(chunk, dt, first);
            }
            memcpy(&mirror[slot], &ht, sizeof(BatchTable));
            ctx->btab_n[slot] = n_items;
        }
        // with given probabilities the counting kernel needs the seeds in place before the first scan
        if (general) seeds_kernel<<<dim3(capped((max_seeds + kBlock - 1) / kBlock, 1 << 20), n_items), kBlock, 0, st>>>(a, dt, dyn);
        for (int h = 1; h <= L; ++h) {
            a.h = h; a.f = general ? 0 : fanouts[h - 1]; a.t = general ? d_t[h - 1] : nullptr;
            const dim3 wgrid(capped((nb[h - 1] * kWave + kBlock - 1) / kBlock, share), n_items);   // a wavefront per target
            if (general) general_count_kernel<<<wgrid, kBlock, 0, st>>>(a, dt);
            // the relabel of the hop before and the emptying of this hop's table ride in the scan's launches
            if (h > 1 && !general) {
                SampleArgs ap = a;
                ap.h = h - 1;
                grid_scan_batched(st, scan_grid, n_items, CountIn{a, dt}, CountOut{a, dt}, CountFin{a, dt}, partial,
                                  RelabelPrev{ap, dt}, TableClear{a, dt});
            } else if (!general) {
                // hop 1: the seeds are put in place by the scan's first launch, which counts from the seeds themselves
                grid_scan_batched_two(st, scan_grid, n_items, CountInSeeds{a, dyn}, CountIn{a, dt}, CountOut{a, dt},
                                      CountFin{a, dt}, partial, SeedsHead{a, dt, dyn}, TableClear{a, dt});
            } else {
                grid_scan_batched(st, scan_grid, n_items, CountIn{a, dt}, CountOut{a, dt}, CountFin{a, dt}, partial,
                                  NoHook(), TableClear{a, dt});
            }
            if (general) {
                general_sample_kernel<<<wgrid, kBlock, 0, st>>>(a, dt);
            } else {
                const int G = a.f <= 8 ? 8 : a.f <= 16 ? 16 : a.f <= 32 ? 32 : 64;
                const dim3 sgrid(capped((nb[h - 1] * G + kBlock - 1) / kBlock, share), n_items);
                switch (G) {
                    case 8:  sample_kernel<8><<<sgrid, kBlock, 0, st>>>(a, dt); break;
                    case 16: sample_kernel<16><<<sgrid, kBlock, 0, st>>>(a, dt); break;
                    case 32: sample_kernel<32><<<sgrid, kBlock, 0, st>>>(a, dt); break;
                    default: sample_kernel<64><<<sgrid, kBlock, 0, st>>>(a, dt); break;
                }
                // hops small enough meet in LDS (the workgroups of the others leave at once); a hop whose bound
                // already exceeds what the partitions hold has no workgroup to launch
                int64_t parts = 1;
                while (parts < (1 << kLdsMaxPartsLog2) && parts * kLdsPartKeys < nb[h - 1] + eb[h]) parts <<= 1;
                dedup_lds_kernel<<<dim3(n_items, (unsigned)parts), kDedupBlock, dedup_lds, st>>>(a, dt);
            }
            grid_scan_batched_two(st, scan_grid, n_items, NewIn{a, dt}, NewInKept{a, dt}, NewOut{a, dt}, NewFin{a, dt}, partial);
            if (h == L || general)
                relabel_kernel<<<dim3(capped((eb[h] + kBlock - 1) / kBlock, share), n_items), kBlock, 0, st>>>(a, dt);
        }
        ctx->sample_flags_clean = 1;
    }
    SPP_HIP(hipGetLastError());
    if (flags & SPP_SYNC) {
        int64_t* hp = ctx->h_pinned + 64;            // kMaxBatches x 18 counts, then the flags
        for (int j = 0; j < n_items; ++j)
            SPP_HIP(hipMemcpyAsync(hp + j * 2 * kE, items[j].io->d_counts, 2 * kE * sizeof(int64_t), hipMemcpyDeviceToHost, st));
        SPP_HIP(hipMemcpyAsync(hp + kMaxBatches * 2 * kE, d_bad, 2 * sizeof(int), hipMemcpyDeviceToHost, st));
        SPP_HIP(hipStreamSynchronize(st));
        for (int j = 0; j < n_items; ++j)
            for (int k = 0; k <= SPP_MAX_L; ++k) {
                items[j].io->n[k] = hp[j * 2 * kE + k];
                items[j].io->e[k] = hp[j * 2 * kE + kE + k];
            }
        const int* fl = reinterpret_cast<const int*>(hp + kMaxBatches * 2 * kE);
        SPP_CHECK((fl[0] & 1) == 0, SPP_E_ARG, "spp_sample_mfg: a seed lies outside [0, N)");
        SPP_CHECK((fl[0] & 2) == 0, SPP_E_ARG, "spp_sample_mfg_general: a transition probability lies outside [0, 1]; it was taken as 0");
        SPP_CHECK((fl[0] & 4) == 0, SPP_E_HIP, "spp_sample_mfg: more than %d ids of one hop share a hash partition; the minibatch's output is not valid", kLdsSlots);
        SPP_CHECK(fl[1] == 0, SPP_E_CAPACITY, "spp_sample_mfg_general: a minibatch exceeded the capacity of its buffers and was abandoned");
    }
    return SPP_OK;
}

extern "C" int spp_sample_mfg_multi(spp_ctx* ctx, const spp_graph* g, const spp_sample_item* items, int32_t n_items,
                                    const int32_t* fanouts, int32_t L, uint64_t seed, uint32_t flags) {
    SPP_CHECK(fanouts, SPP_E_ARG, "spp_sample_mfg: null argument");
    return sample_batches(ctx, g, items, n_items, fanouts, nullptr, L, seed, flags);
}

extern "C" int spp_sample_mfg_general(spp_ctx* ctx, const spp_graph* g, const float* const* d_t,
                                      const spp_sample_item* items, int32_t n_items, int32_t L, uint64_t seed,
                                      uint32_t flags) {
    SPP_CHECK(d_t, SPP_E_ARG, "spp_sample_mfg_general: null argument");
    return sample_batches(ctx, g, items, n_items, nullptr, d_t, L, seed, flags);
}

extern "C" int spp_sample_mfg(spp_ctx* ctx, const spp_graph* g, const int32_t* d_seeds, int32_t nseeds,
                              const int32_t* fanouts, int32_t L, uint64_t seed, uint64_t batch_index,
                              spp_mfg* io, uint32_t flags) {
    SPP_CHECK(io, SPP_E_ARG, "spp_sample_mfg: null argument");
    spp_sample_item one;
    one.d_seeds = d_seeds; one.nseeds = nseeds; one.batch_index = batch_index; one.io = io;
    return spp_sample_mfg_multi(ctx, g, &one, 1, fanouts, L, seed, flags);
}
