// Node-wise fanout sampling into per-layer message-flow graphs (Sec. 2.3; the process of Sec. 3.1).
//
// Per hop h, all on the context's stream with every count kept on the device:
//   1. grid scan of c_i = min(f_h, d(S_{h-1}[i]))            -> indptr of MFG h, e_h
//   2. sample: a group of G lanes (G = 8/16/32/64 >= f_h) per target draws its slots in parallel
//      (one Philox block per lane), resolves Floyd's "already taken" rule with ballots, reads the
//      neighbour ids and offers (id, n_{h-1} + flat position) to the id table with atomic min
//   3. grid scan of "this flat entry is the first appearance of a new id"
//                                                            -> S_h appended in order, n_h, table value := local id
//   4. relabel: src[e] = table value of the e-th sampled id
// The table (open addressing, global memory, sized for the bound on |S_L|) lives for the whole
// batch: after hop h every key's value is its index in S_h, which is below any position offered
// at hop h+1, so earlier vertices keep their ids.
#include "spp_common.h"
#include "spp_device.h"

namespace spp {

struct SampleArgs {
    const int64_t* rowptr;
    const int32_t* col;
    int64_t        N;
    unsigned long long* tab;
    uint32_t       mask;
    int            shift;
    int32_t*       S;          // node ids
    int32_t*       indptr;     // this hop
    int32_t*       src;        // this hop
    int32_t*       flat;       // sampled global ids of this hop
    int64_t*       counts;     // n[0..MAX_L], e[0..MAX_L]
    unsigned long long* totals; // context-wide running sums: [0] batches, [1] |S_L|, [2] edges
    int            L;
    int            h;          // hop, 1-based
    int            f;          // fanout of this hop
    uint64_t       seed;
    uint32_t       batch_lo;
};

__device__ __forceinline__ const int64_t* n_ptr(const SampleArgs& a, int h) { return a.counts + h; }
__device__ __forceinline__ const int64_t* e_ptr(const SampleArgs& a, int h) { return a.counts + (SPP_MAX_L + 1) + h; }

// Empties the id table and zeroes the counts and the error flag of a new batch.
__global__ void __launch_bounds__(kBlock) sample_init_kernel(SampleArgs a, int64_t cap, int nseeds, int* __restrict__ bad) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    for (int64_t i = t; i < cap; i += stride) a.tab[i] = ~0ull;
    if (t == 0) {
        for (int k = 0; k <= SPP_MAX_L; ++k) { a.counts[k] = 0; a.counts[SPP_MAX_L + 1 + k] = 0; }
        a.counts[0] = nseeds;
        *bad = 0;
    }
}

__global__ void __launch_bounds__(kBlock) seeds_kernel(SampleArgs a, const int32_t* __restrict__ seeds, int nseeds,
                                                       int* __restrict__ bad) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= nseeds) return;
    int32_t v = seeds[i];
    if (v < 0 || v >= a.N) { v = 0; atomicOr(bad, 1); }       // reported; keeps later row reads in range
    a.S[i] = v;
    table_insert_min(a.tab, a.mask, a.shift, (uint32_t)v, (uint32_t)i);
}

// ---- step 1 ----
struct CountIn {
    SampleArgs a;
    __device__ int operator()(int64_t i) const {
        const int64_t v = a.S[i];
        const int64_t d = a.rowptr[v + 1] - a.rowptr[v];
        return (int)(d < a.f ? d : a.f);
    }
};
struct CountOut {
    SampleArgs a;
    __device__ void operator()(int64_t i, int ex, int) const { a.indptr[i] = ex; }
};
struct CountFin {
    SampleArgs a;
    __device__ void operator()(int total) const {
        a.indptr[a.counts[a.h - 1]] = total;
        a.counts[SPP_MAX_L + 1 + a.h] = total;
        atomicAdd(&a.totals[2], (unsigned long long)(uint32_t)total);
    }
};

// ---- step 2 ----
template <int G>
__global__ void __launch_bounds__(kBlock) sample_kernel(SampleArgs a) {
    const int lane = lane_id();
    const int j = lane & (G - 1);                  // slot handled by this lane
    const int gbase = lane - j;                    // first lane of the group inside the wavefront
    const uint64_t gmask = (G == 64) ? ~0ull : (((1ull << (G & 63)) - 1ull) << gbase);
    constexpr int kGroupsPerWave = kWave / G;
    const int64_t n_prev = *n_ptr(a, a.h - 1);
    const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    const int f = a.f;

    for (int64_t first = wave * kGroupsPerWave; first < n_prev; first += nwaves * kGroupsPerWave) {
        const int64_t i = first + (lane / G);
        const bool valid = i < n_prev;
        int64_t r0 = 0, d = 0;
        int32_t off = 0, v = 0;
        if (valid) {
            v = a.S[i];
            r0 = a.rowptr[v];
            d = a.rowptr[v + 1] - r0;
            off = a.indptr[i];
        }
        const bool floyd = d > f;
        const int c = floyd ? f : (int)d;
        int64_t pos = j;                           // d <= f: the whole row, in row order
        if (floyd) {
            // Floyd's subset algorithm, one draw per slot: m = d - f + j, t uniform on [0, m]
            const uint64_t m = (uint64_t)(d - f + j);
            uint64_t t = 0;
            if (j < f) {
                const uint32_t r = rand32(a.seed, a.batch_lo, (uint32_t)a.h, (uint32_t)v, (uint32_t)j);
                t = ((uint64_t)r * (m + 1ull)) >> 32;
            }
            pos = (int64_t)t;
            // slot jj takes t_jj unless an earlier slot already holds it, else m_jj (never held before)
            for (int jj = 1; jj < f; ++jj) {
                const int64_t tj = __shfl((long long)t, gbase + jj, kWave);
                const bool hit = (j < jj) && (pos == tj);
                const uint64_t b = __ballot(hit) & gmask;
                if (j == jj && b != 0ull) pos = (int64_t)m;
            }
        }
        if (valid && j < c) {
            const int32_t gid = a.col[r0 + pos];
            const int64_t e = (int64_t)off + j;
            a.flat[e] = gid;
            table_insert_min(a.tab, a.mask, a.shift, (uint32_t)gid, (uint32_t)(n_prev + e));
        }
    }
}

// ---- step 3 ----
struct NewIn {
    SampleArgs a;
    __device__ int operator()(int64_t e) const {
        uint32_t val = 0;
        table_find(a.tab, a.mask, a.shift, (uint32_t)a.flat[e], val);
        return (int64_t)val == a.counts[a.h - 1] + e ? 1 : 0;
    }
};
struct NewOut {
    SampleArgs a;
    __device__ void operator()(int64_t e, int ex, int v) const {
        if (!v) return;
        const uint32_t gid = (uint32_t)a.flat[e];
        uint32_t val = 0;
        const int64_t slot = table_find(a.tab, a.mask, a.shift, gid, val);
        const int64_t id = a.counts[a.h - 1] + ex;
        a.S[id] = (int32_t)gid;
        // the new value is <= the old one and is never equal to another entry's own position, so
        // threads still testing "first appearance" read either value with the same outcome
        __hip_atomic_store(&a.tab[slot], ((unsigned long long)gid << 32) | (uint32_t)id, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
};
struct NewFin {
    SampleArgs a;
    __device__ void operator()(int total) const {
        const int64_t n = a.counts[a.h - 1] + total;
        a.counts[a.h] = n;
        if (a.h == a.L) { atomicAdd(&a.totals[1], (unsigned long long)n); atomicAdd(&a.totals[0], 1ull); }
    }
};

// ---- step 4 ----
__global__ void __launch_bounds__(kBlock) relabel_kernel(SampleArgs a) {
    const int64_t e_h = *e_ptr(a, a.h);
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < e_h; e += stride) {
        uint32_t val = 0;
        table_find(a.tab, a.mask, a.shift, (uint32_t)a.flat[e], val);
        a.src[e] = (int32_t)val;
    }
}

template <int G>
static void launch_sample(int grid, hipStream_t st, const SampleArgs& a) {
    sample_kernel<G><<<grid, kBlock, 0, st>>>(a);
}

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

extern "C" int spp_sample_mfg(spp_ctx* ctx, const spp_graph* g, const int32_t* d_seeds, int32_t nseeds,
                              const int32_t* fanouts, int32_t L, uint64_t seed, uint64_t batch_index,
                              spp_mfg* io, uint32_t flags) {
    using namespace spp;
    SPP_CHECK(ctx && g && fanouts && io, SPP_E_ARG, "spp_sample_mfg: null argument");
    SPP_CHECK(nseeds >= 0 && (d_seeds || nseeds == 0), SPP_E_ARG, "spp_sample_mfg: seeds");
    int64_t nb[SPP_MAX_L + 1], eb[SPP_MAX_L + 1];
    SPP_TRY(spp_mfg_bound(nseeds, fanouts, L, g->N, nb, eb));
    SPP_CHECK(nseeds <= g->N, SPP_E_ARG, "spp_sample_mfg: more seeds than vertices");
    SPP_CHECK(io->d_node_ids && io->d_counts, SPP_E_ARG, "spp_sample_mfg: null output buffer");
    SPP_CHECK(io->n_nodes_cap >= nb[L] && io->n_nodes_cap >= 1, SPP_E_CAPACITY,
              "spp_sample_mfg: d_node_ids holds %lld entries, the bound is %lld", (long long)io->n_nodes_cap, (long long)nb[L]);
    int64_t emax = 1;
    for (int h = 1; h <= L; ++h) {
        SPP_CHECK(io->d_indptr[h - 1] && io->d_src[h - 1], SPP_E_ARG, "spp_sample_mfg: null buffer of hop %d", h);
        SPP_CHECK(io->n_edges_cap[h - 1] >= eb[h], SPP_E_CAPACITY, "spp_sample_mfg: d_src of hop %d holds %lld entries, the bound is %lld",
                  h, (long long)io->n_edges_cap[h - 1], (long long)eb[h]);
        SPP_CHECK(eb[h] < 0x7FFFFFFFll && nb[h] + eb[h] < 0xFFFFFFFFll, SPP_E_ARG, "spp_sample_mfg: hop %d exceeds 32-bit offsets", h);
        if (eb[h] > emax) emax = eb[h];
    }
    SPP_HIP(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;

    const uint32_t cap = next_pow2((uint64_t)(2 * nb[L] > 1024 ? 2 * nb[L] : 1024));
    int shift = 32;
    for (uint32_t c = cap; c > 1; c >>= 1) --shift;
    const int scan_grid = ctx->num_cu * 4;
    SPP_TRY(ctx->table.reserve((size_t)cap * sizeof(uint64_t)));
    SPP_TRY(ctx->flat.reserve((size_t)emax * sizeof(int32_t)));
    SPP_TRY(ctx->partials.reserve((size_t)scan_grid * sizeof(int) + 64));
    int* partial = ctx->partials.as<int>();
    int* d_bad = partial + scan_grid;

    SampleArgs a;
    a.rowptr = g->rowptr; a.col = g->col; a.N = g->N;
    a.tab = ctx->table.as<unsigned long long>(); a.mask = cap - 1; a.shift = shift;
    a.S = io->d_node_ids; a.flat = ctx->flat.as<int32_t>(); a.counts = io->d_counts;
    a.seed = seed; a.batch_lo = (uint32_t)batch_index;
    a.totals = reinterpret_cast<unsigned long long*>(ctx->totals); a.L = L;
    a.indptr = nullptr; a.src = nullptr; a.h = 0; a.f = 0;

    {
        ScopedTimer tt(ctx, SPP_T_SAMPLE, st);
        const int fill_grid = (int)((cap / kBlock) < (uint32_t)(ctx->num_cu * 8) ? (cap / kBlock) : (uint32_t)(ctx->num_cu * 8));
        sample_init_kernel<<<fill_grid > 0 ? fill_grid : 1, kBlock, 0, st>>>(a, (int64_t)cap, nseeds, d_bad);
        if (nseeds > 0) seeds_kernel<<<(nseeds + kBlock - 1) / kBlock, kBlock, 0, st>>>(a, d_seeds, nseeds, d_bad);
        for (int h = 1; h <= L; ++h) {
            a.h = h; a.f = fanouts[h - 1];
            a.indptr = io->d_indptr[h - 1];
            a.src = io->d_src[h - 1];
            grid_scan(st, scan_grid, a.counts + (h - 1), CountIn{a}, CountOut{a}, CountFin{a}, partial);
            const int G = a.f <= 8 ? 8 : a.f <= 16 ? 16 : a.f <= 32 ? 32 : 64;
            int64_t need = (nb[h - 1] * G + kBlock - 1) / kBlock;
            const int grid = (int)(need < (int64_t)ctx->num_cu * 16 ? (need > 0 ? need : 1) : (int64_t)ctx->num_cu * 16);
            switch (G) {
                case 8:  launch_sample<8>(grid, st, a); break;
                case 16: launch_sample<16>(grid, st, a); break;
                case 32: launch_sample<32>(grid, st, a); break;
                default: launch_sample<64>(grid, st, a); break;
            }
            grid_scan(st, scan_grid, a.counts + (SPP_MAX_L + 1) + h, NewIn{a}, NewOut{a}, NewFin{a}, partial);
            int64_t rneed = (eb[h] + kBlock - 1) / kBlock;
            const int rgrid = (int)(rneed < (int64_t)ctx->num_cu * 8 ? (rneed > 0 ? rneed : 1) : (int64_t)ctx->num_cu * 8);
            relabel_kernel<<<rgrid, kBlock, 0, st>>>(a);
        }
    }
    SPP_HIP(hipGetLastError());
    if (flags & SPP_SYNC) {
        int64_t* hp = ctx->h_pinned;
        SPP_HIP(hipMemcpyAsync(hp, io->d_counts, 2 * (SPP_MAX_L + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, st));
        SPP_HIP(hipMemcpyAsync(hp + 32, d_bad, sizeof(int), hipMemcpyDeviceToHost, st));
        SPP_HIP(hipStreamSynchronize(st));
        for (int k = 0; k <= SPP_MAX_L; ++k) { io->n[k] = hp[k]; io->e[k] = hp[SPP_MAX_L + 1 + k]; }
        SPP_CHECK(*reinterpret_cast<int*>(hp + 32) == 0, SPP_E_ARG, "spp_sample_mfg: a seed lies outside [0, N)");
    }
    return SPP_OK;
}
