/*
 * spp.h -- C interface of the per-partition data path of VIP-cached, partitioned GNN
 * minibatch preparation on one AMD MI355X (gfx950):
 *
 *   spp_vip_propagate     vertex-inclusion probabilities, Proposition 1 (Sec. 3.1)
 *   spp_build_vip_cache   VIP-ranked replica cache of remote feature rows (Secs. 3.2, 4.2)
 *   spp_sample_mfg        node-wise fanout sampling into per-layer message-flow graphs
 *                         (Sec. 2.3; steps (i)-(iii) of the random process of Sec. 3.1)
 *   spp_gather_features   cache-aware feature gather: local shard / replica cache / remote
 *                         rows on a miss (Secs. 4.1-4.3; stages 5-10 of Appendix D)
 *
 * Conventions
 *   G        directed graph in CSR on the device: rowptr int64[N+1], col int32[M].  Row v,
 *            adj(v) = col[rowptr[v] .. rowptr[v+1]), is the list v samples its neighbours
 *            from; d(v) = |adj(v)|.  Rows ascending, duplicate-free, no self loops.
 *   T        training vertices of the owned partition (device int32, distinct).
 *   fanouts  host int32[L]; fanouts[h-1] = f_h, hop h = 1 being the hop next to the minibatch.
 *   [lo,hi)  the owned partition's contiguous vertex-id range (Sec. 4.1).
 *   K, alpha number of partitions and replication factor: the cache holds at most
 *            floor(alpha * N / K) rows (Sec. 3.2).
 *   remote store: the feature matrix with the owned range cut out, row-major;
 *            row of vertex g = g if g < lo, else g - (hi - lo).
 *
 * Pointers named d_* are device memory, host_* pinned (device-mapped) host memory unless
 * said otherwise; the rest is ordinary host memory.  The caller owns every buffer it passes;
 * the library owns only what lives behind its opaque handles.  All device work is enqueued
 * on the context's stream (the miss path of the gather also uses a side stream owned by the
 * context and joins it back before returning).  Calls on one context must not overlap.
 *
 * Every function returns SPP_OK (0) or a negative code; spp_last_error() then describes it.
 * Nothing here throws, aborts or falls back to the CPU.
 */
#ifndef SPP_H
#define SPP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPP_MAX_L       8      /* most hops / GNN layers */
#define SPP_MAX_FANOUT  64     /* largest fanout (one wavefront lane per slot) */
#define SPP_MAX_GATHER_LISTS 64 /* most id lists in one spp_gather_features_multi call */
#define SPP_MAX_SAMPLE_BATCHES 64 /* most minibatches in one spp_sample_mfg_multi call */
#define SPP_STATIC_GATHER_MAX_ROWS 131072 /* most ids in one spp_gather_features_static call */

enum {
    SPP_OK          =  0,
    SPP_E_ARG       = -1,      /* null pointer, size out of range, misaligned rows, L or fanout too large */
    SPP_E_CAPACITY  = -2,      /* an output buffer is smaller than the bound the call needs */
    SPP_E_OOM       = -3,      /* device or host allocation failed */
    SPP_E_HIP       = -4       /* a HIP runtime call failed (text in spp_last_error) */
};

/* flags */
#define SPP_SYNC              0x1u   /* wait for the stream before returning and fill host outputs */
#define SPP_VIP_INCLUDE_HOP0  0x2u   /* also multiply (1 - p^[0]) into eq. (1); default: as printed, h = 1..L */
#define SPP_GRAPH_IN_LISTS    0x4u   /* spp_graph_create: also build the transposed edge structure (who can sample u)
                                        that vip_propagate needs: 4 bytes per edge of device memory */
#define SPP_GRAPH_CHUNKED     0x20u  /* spp_graph_create, with SPP_GRAPH_IN_LISTS: build the layout for graphs whose
                                        per-vertex vectors exceed the caches (two passes per dense hop) whatever N is;
                                        by default graphs above 2^23 vertices get it */
#define SPP_SAMPLE_GLOBAL_TABLE 0x40u /* spp_sample_mfg(_multi): deduplicate every hop through the id table in global memory,
                                        also the hops small enough for the LDS form (same results; for comparison and tests) */
#define SPP_NO_JOIN           0x8u   /* gather: leave the miss copy running on the side stream; see spp_gather_join */
#define SPP_STORE_ORDER       0x10u  /* gather: fetch the call's missed remote rows in the order of the remote store;
                                        see spp_gather_features_multi */
#define SPP_HIT_BESIDE_MISS   0x80u  /* gather, with SPP_NO_JOIN in a loop of calls: queue this call's miss copy before
                                        its hit copy, so that it starts the moment the miss copy of the call before
                                        ends and the host link never idles; the hit copy then runs beside it on the
                                        CUs it leaves free (same results; higher pipeline rate, slower hit copy) */

typedef struct spp_ctx   spp_ctx;    /* workspaces, side stream, events */
typedef struct spp_graph spp_graph;  /* refers to the caller's CSR; owns the library-built transposed structure */
typedef struct spp_cache spp_cache;  /* owns the id->slot table and the cached rows in HBM */

/* Thread-local description of the last error on this thread; valid until the next call. */
const char* spp_last_error(void);

/* Creates a context on `device`; `hip_stream` is the caller's hipStream_t (NULL = the null
 * stream).  The caller keeps the stream alive until spp_ctx_destroy. */
int  spp_ctx_create(spp_ctx** out, int device, void* hip_stream);
void spp_ctx_destroy(spp_ctx* ctx);
/* Blocks until everything the context enqueued has finished. */
int  spp_ctx_sync(spp_ctx* ctx);

/* Wraps a device CSR (not copied; must outlive the handle).  With SPP_GRAPH_IN_LISTS it also
 * builds, once, the transposed structure (the edges v -> u grouped by blocks of destination
 * vertices u and sorted by v inside a block: who can sample u), which costs about
 * 4*M + N/64 bytes of device memory plus 16*M bytes of temporary space while it is built.
 * Synchronous. */
int  spp_graph_create(spp_ctx* ctx, int64_t N, int64_t M, const int64_t* d_rowptr,
                      const int32_t* d_col, uint32_t flags, spp_graph** out);
void spp_graph_destroy(spp_graph* g);

/* (1) Vertex-inclusion probabilities, Proposition 1 with the uniform instantiation of Sec. 3.1:
 *       p^[0](u) = min(1, B/nT) for u in T, else 0
 *       p^[h](u) = 1 - prod over {v : u in adj(v)} of (1 - min(1, f_h/d(v)) * p^[h-1](v))    eq. (2)
 *       p(u)     = 1 - prod_{h=1..L} (1 - p^[h](u))                                         eq. (1)
 *     Products are carried as sums of log1p in fp64; results are stored as fp32.  The call waits
 *     for the device at most once per hop (it reads the size of the hop's frontier to choose
 *     between the push and the pull form), and not at all after the first pulled hop: the hops
 *     that follow are pulled without asking.
 *     d_p_total: fp32[N], required.  d_p_hop: fp32[L*N] (hop h at offset (h-1)*N) or NULL.
 *     flags: SPP_VIP_INCLUDE_HOP0, SPP_SYNC.  The graph must have been created with
 *     SPP_GRAPH_IN_LISTS (else SPP_E_ARG).  Vertices with d(v) = 0 contribute nothing. */
int  spp_vip_propagate(spp_ctx* ctx, const spp_graph* g, const int32_t* d_T, int64_t nT,
                       int32_t B, const int32_t* fanouts, int32_t L,
                       float* d_p_total, float* d_p_hop, uint32_t flags);

/* How the last spp_vip_propagate on this context walked each hop: pushed[h-1] = 1 if hop h was done
 * in push form over a sparse frontier (its out-edges were at most M/16), 0 if it was pulled over
 * the transposed structure; frontier_edges[h-1] = out-edges of the vertices with a non-zero weight at hop h
 * (the edges a hop has to touch at all), or -1 where the library did not ask: the hop after a pulled
 * hop is pulled too.  Either array may be NULL. */
int  spp_vip_last_hops(spp_ctx* ctx, int32_t* pushed, int64_t* frontier_edges, int32_t L);

/* (2) Replica cache (Sec. 3.2): among the vertices outside [lo,hi) with d_score > 0, the first
 *     C = floor(alpha*N/K) in the order (score descending as fp32, id ascending); slot = rank.
 *     d_score fp32[N] is the VIP vector (or any other ranking score, e.g. degree).
 *     Writes the ids in rank order to d_cache_ids (device, capacity >= C) and their number to
 *     *n_cached (host), builds the id->slot hash table (Sec. 4.2) and copies the chosen rows once
 *     from the remote store (pinned host memory, or device memory) into HBM.  remote may be
 *     NULL: then no rows are copied and the cache only answers membership (spp_cache_lookup).
 *     Row size D*elem_bytes must be a multiple of 2.  Synchronous. */
int  spp_build_vip_cache(spp_ctx* ctx, const float* d_score, int64_t N, int64_t lo, int64_t hi,
                         int32_t K, double alpha, const void* remote, int32_t D,
                         int32_t elem_bytes, int32_t* d_cache_ids, int64_t* n_cached,
                         spp_cache** out);
void spp_cache_destroy(spp_cache* c);
/* Limits the cache to its first `n_slots` ranks (the cache of a smaller alpha is a prefix of a
 * larger one); n_slots < 0 restores all built rows. */
int  spp_cache_set_limit(spp_cache* c, int64_t n_slots);
/* d_slot_out[i] = slot of d_ids[i] in the cache, or -1.  Enqueued on the context's stream. */
int  spp_cache_lookup(spp_ctx* ctx, const spp_cache* c, const int32_t* d_ids, int64_t n,
                      int32_t* d_slot_out);

/* (3) Sampling.  S_0 = seeds (device int32[nseeds], distinct).  At hop h every vertex v of
 *     S_{h-1}, in order, takes c = min(f_h, d(v)) positions of adj(v): all of them in row order
 *     if d(v) <= f_h, otherwise Floyd's subset algorithm with one draw per slot j: m = d-f+j,
 *     t = (rand32 * (m+1)) >> 32, position t unless already taken, else m.  rand32 is word j%4 of
 *     Philox-4x32-10 with key (seed low, seed high) and counter (v, j/4, h, batch_index low).
 *     S_h = S_{h-1} followed by the ids not seen before in order of first appearance (target-
 *     major, slot-minor).  MFG h has targets S_{h-1} and sources S_h: d_indptr[h-1] holds
 *     n_{h-1}+1 offsets, d_src[h-1] the index in S_h of each sampled neighbour; the message of
 *     edge e flows from source d_src[h-1][e] to its target.
 *
 *     The caller sizes the buffers with spp_mfg_bound and fills the capacities and pointers;
 *     the library fills the buffers and d_counts (device int64[2*(SPP_MAX_L+1)]: n_0..n_L at
 *     [0..L], e_0..e_L at [SPP_MAX_L+1 ..]; e_0 = 0).  With SPP_SYNC it also waits and fills the
 *     host fields n[] and e[].  Capacities below the bounds give SPP_E_CAPACITY before any work. */
typedef struct {
    int64_t  n_nodes_cap;               /* in: entries in d_node_ids (>= n_bound[L]) */
    int64_t  n_edges_cap[SPP_MAX_L];    /* in: entries in d_src[h-1] (>= e_bound[h]) */
    int32_t* d_node_ids;                /* out: S_L; its first n[h] entries are S_h */
    int32_t* d_indptr[SPP_MAX_L];       /* out: hop h at [h-1], int32[n_bound[h-1] + 1] */
    int32_t* d_src[SPP_MAX_L];          /* out: hop h at [h-1] */
    int64_t* d_counts;                  /* out: device int64[2*(SPP_MAX_L+1)] */
    int64_t  n[SPP_MAX_L + 1];          /* out (host, with SPP_SYNC): |S_h| */
    int64_t  e[SPP_MAX_L + 1];          /* out (host, with SPP_SYNC): edges of hop h */
} spp_mfg;

/* n_bound[h] = min(N, n_bound[h-1] * (1 + f_h)), e_bound[h] = n_bound[h-1] * f_h; arrays of L+1. */
int  spp_mfg_bound(int32_t nseeds, const int32_t* fanouts, int32_t L, int64_t N,
                   int64_t* n_bound, int64_t* e_bound);
int  spp_sample_mfg(spp_ctx* ctx, const spp_graph* g, const int32_t* d_seeds, int32_t nseeds,
                    const int32_t* fanouts, int32_t L, uint64_t seed, uint64_t batch_index,
                    spp_mfg* io, uint32_t flags);

/* The same sampling for up to SPP_MAX_SAMPLE_BATCHES minibatches in one set of launches (every kernel
 * gets a second grid dimension that names the minibatch; each minibatch has its own id table and
 * counts and its own caller-provided spp_mfg, so results are those of one call per minibatch).
 * A single minibatch of B = 1024 seeds cannot fill 256 CUs, and its dependent launches are latency-bound;
 * sampling the minibatches a pipeline keeps in flight together spreads that latency over all of them. */
typedef struct {
    const int32_t* d_seeds;
    int32_t        nseeds;
    uint64_t       batch_index;
    spp_mfg*       io;
} spp_sample_item;
int  spp_sample_mfg_multi(spp_ctx* ctx, const spp_graph* g, const spp_sample_item* items, int32_t n_items,
                          const int32_t* fanouts, int32_t L, uint64_t seed, uint32_t flags);

/* (4) Gather: d_out[i,:] = row of vertex d_node_ids[i] (in [0, N)), i < n, taken from
 *       d_local  [hi-lo, D]  if lo <= g < hi            (row g - lo)
 *       the cache             if g is cached             (row = slot)
 *       remote                otherwise, a miss          (row g, or g - (hi-lo) above the range)
 *     Hits are copied by one kernel on the context's stream; the compacted miss list is served
 *     by a second kernel on the context's side stream reading the pinned host rows directly,
 *     and joined back before the call returns to the stream.  cache may be NULL (alpha = 0).
 *     n (at most 2^26) is the number of ids, or an upper bound when d_n (device int64, e.g.
 *     &d_counts[L]) is given, in which case the count is read on the device.  Row size D*elem_bytes must be a
 *     multiple of 2 and every store and output 2-byte aligned (SPP_E_ARG otherwise); 16-byte
 *     multiples and alignments take the widest path.  Duplicate ids are allowed.
 *     `remote` is pinned host memory (or device memory); it may be NULL only if no id misses.
 *     stats (host, may be NULL) is filled when SPP_SYNC is set; otherwise read it later with
 *     spp_gather_last_stats after synchronising. */
/* n_local counts every id of the owned range; n_local_host of them were read from host memory
 * (only with a split local store, see spp_build_local_store).  n_miss counts every row that is
 * neither local nor cached; in a call with several lists a remote vertex that several rows miss
 * is read from the remote store once and copied to the other rows on the device: n_miss_shared
 * of the n_miss rows were served that way.  miss_bytes = bytes read from host memory
 * = (n_miss - n_miss_shared + n_local_host) * row size. */
typedef struct { int64_t n_local, n_cache_hit, n_miss, miss_bytes, n_local_host, n_miss_shared; } spp_gather_stats;
int  spp_gather_features(spp_ctx* ctx, const spp_cache* cache, const void* d_local,
                         int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D, int32_t elem_bytes,
                         const int32_t* d_node_ids, int64_t n, const int64_t* d_n, void* d_out,
                         spp_gather_stats* stats, uint32_t flags);
int  spp_gather_last_stats(spp_ctx* ctx, spp_gather_stats* stats);
/* spp_gather_features for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, results and statistics as
 * spp_gather_features, same kernels; the per-call workspace (counters, one source descriptor per id,
 * the hit and miss lists: 28 bytes per id) lives in a fixed array of the library's device image,
 * 3.5 MB on every GPU the library runs on until the process ends, instead of the context's
 * grow-only buffers, and the call makes no hipMalloc / hipFree and creates no events.
 * Limits: n <= SPP_STATIC_GATHER_MAX_ROWS (SPP_E_ARG beyond, before any work); flags SPP_SYNC only
 * (SPP_STORE_ORDER needs a table per remote row, SPP_NO_JOIN would leave the shared workspace in
 * use: both SPP_E_ARG); the miss copy is joined before the call returns to the stream; the call is
 * left out of the timing report.  A gather that an earlier call on the context left unjoined is
 * joined first.  Every call on a GPU uses that GPU's one array, whichever context it comes from:
 * calls on different streams that overlap on one GPU race and must be ordered by the caller. */
int  spp_gather_features_static(spp_ctx* ctx, const spp_cache* cache, const void* d_local,
                                int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D, int32_t elem_bytes,
                                const int32_t* d_node_ids, int64_t n, const int64_t* d_n, void* d_out,
                                spp_gather_stats* stats, uint32_t flags);
/* With SPP_NO_JOIN a gather returns to the context's stream as soon as the hit copy is enqueued,
 * while the missed rows are still arriving on the side stream; work enqueued next on the stream
 * (the sampling of the following minibatches) overlaps the PCIe transfer.  spp_gather_join makes
 * the stream wait for that miss copy and then copies the rows that share a fetched vertex with
 * another row of the call: call it before anything that reads the gathered rows.  The next
 * gather on the same context, spp_ctx_sync and SPP_SYNC join by themselves.  Until the join
 * has run, the id lists and the outputs of the call must stay allocated: the side stream and
 * the join still write them. */
int  spp_gather_join(spp_ctx* ctx);

/* The same gather for up to SPP_MAX_GATHER_LISTS id lists in one set of launches (one
 * classification, one hit copy, one miss copy), e.g. the minibatches a pipeline keeps in flight
 * (Sec. 4.3 keeps ten): each kernel then moves several minibatches' worth of rows per launch.
 * List j: d_out[i,:] = row of vertex d_node_ids[i], i < n (n an upper bound when d_n is given).
 * The statistics are summed over the lists.
 * A remote vertex that several rows of the call miss is read from the remote store once
 * (n_miss_shared counts the other rows, which are copied on the device).
 * SPP_STORE_ORDER changes how that is done, never the result: the missed vertices are marked in an
 * array with one entry per row of the remote store (4 bytes each, cleared and scanned per call)
 * and fetched in the store's order, so that rows that are neighbours in the store share the
 * memory lines they straddle.  It pays when a call misses a sizeable share of the store (an
 * eighth or more: then the fetch is 3 to 15 % faster) and costs a pass over that array
 * otherwise.
 * SPP_HIT_BESIDE_MISS changes the order of the call's two copies, never the result: by default the
 * stream waits for the miss copy of the call before, copies the hits with the whole chip and then
 * starts this call's miss copy; with the flag the miss copy is queued first (it starts when the
 * earlier one ends) and the hit copy runs beside it.  It pays in a loop of SPP_NO_JOIN calls whose
 * hit copy takes a sizeable part of the time between two miss copies.
 * flags: SPP_SYNC, SPP_NO_JOIN, SPP_STORE_ORDER, SPP_HIT_BESIDE_MISS. */
typedef struct {
    const int32_t* d_node_ids;
    int64_t        n;
    const int64_t* d_n;      /* device int64 count, or NULL */
    void*          d_out;    /* [n, D] */
} spp_gather_list;
int  spp_gather_features_multi(spp_ctx* ctx, const spp_cache* cache, const void* d_local,
                               int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D,
                               int32_t elem_bytes, const spp_gather_list* lists, int32_t n_lists,
                               spp_gather_stats* stats, uint32_t flags);

/* (f) VIP-ordered local storage (Sec. 3.2, paragraph on host-to-device transfer reduction; Sec. 4.1;
 *     Sec. 5, local partition storage on CPU versus GPU).  The partition's own vertices [lo, hi) are
 *     ranked by (d_score descending, id ascending; a score that is not positive counts as 0, so a
 *     constant score gives the id order) and the rows of the first floor(beta * (hi-lo)) of that
 *     order are copied into device memory, in rank order; the other local rows are read from
 *     local_rows when a gather needs them, on the miss path (side stream), like remote misses.
 *     local_rows [hi-lo, D] (row g - lo) is pinned host memory (or device memory) owned by the
 *     caller; it must stay valid while the store is used.  The store keeps a device array
 *     int32[hi-lo] with every local vertex's rank (the paper renumbers the vertices instead).
 *     n_device_rows (host, out) = rows kept in device memory.
 *     spp_local_store_set_limit: use only the first n_rows of the device rows (a smaller beta is a
 *     prefix of a larger one); negative = all.
 *     spp_local_store_rank: d_rank_out[i] = rank of d_ids[i], or -1 if it is not in [lo, hi). */
typedef struct spp_local_store spp_local_store;
int  spp_build_local_store(spp_ctx* ctx, const float* d_score, int64_t N, int64_t lo, int64_t hi, double beta,
                           const void* local_rows, int32_t D, int32_t elem_bytes,
                           int64_t* n_device_rows, spp_local_store** out);
void spp_local_store_destroy(spp_local_store* store);
int  spp_local_store_set_limit(spp_local_store* store, int64_t n_rows);
int  spp_local_store_rank(spp_ctx* ctx, const spp_local_store* store, const int32_t* d_ids, int64_t n,
                          int32_t* d_rank_out);
/*     The gather of spp_gather_features_multi with the local shard held by such a store: a local
 *     id whose rank is below the limit is copied from the device rows by the hit kernel, any other
 *     local id joins the miss list and is read from local_rows.  Results are byte-identical to
 *     the gather with the whole shard in device memory. */
int  spp_gather_features_split(spp_ctx* ctx, const spp_cache* cache, const spp_local_store* store,
                               int64_t N, int64_t lo, int64_t hi, const void* remote, int32_t D,
                               int32_t elem_bytes, const spp_gather_list* lists, int32_t n_lists,
                               spp_gather_stats* stats, uint32_t flags);

/* (f) Proposition 1 with arbitrary probabilities (Sec. 3.1, paragraph after the proposition: any
 *     initial sampling and any hop-wise transition probability function):
 *       d_p0   device fp32[N]: probability that v is in the minibatch
 *       d_t    HOST array of L device pointers; d_t[h-1] is fp32[M], aligned with the CSR's col:
 *              the probability that the vertex of the row samples that entry at hop h
 *       p^[h](u) = 1 - prod over edges e with col[e] = u of (1 - d_t[h-1][e] * p^[h-1](row(e)))
 *     and p(u) as in eq. (1).  Walked in push form over the CSR (the graph needs no transposed
 *     structure), fp64 log-sums, fp32 results; no host synchronisation inside.  On a graph
 *     created with SPP_GRAPH_IN_LISTS the edges' terms go through per-row-block bins instead of
 *     global atomic adds (about four times faster); the terms are then formed and held in fp32
 *     (a few ulp each, all of one sign, so the sums keep that relative accuracy) and the context
 *     keeps 8*M bytes of device memory for the bins.  A probability outside [0, 1] (or not a
 *     number) counts as 0 and is reported (SPP_E_ARG) when SPP_SYNC is set.
 *     flags: SPP_VIP_INCLUDE_HOP0, SPP_SYNC. */
int  spp_vip_propagate_general(spp_ctx* ctx, const spp_graph* g, const float* d_p0, const float* const* d_t,
                               int32_t L, float* d_p_total, float* d_p_hop, uint32_t flags);

/*     A sampler whose transition probabilities are exactly d_t: at hop h a target v takes every
 *     entry of its row independently, entry k (edge e) iff
 *       rand32(seed, batch_index, h, v, k) < floor(d_t[h-1][e] * 2^32)   (64-bit comparison),
 *     so a target's sample has no fixed size.  Layout, relabelling, batching over several
 *     minibatches and the random stream are those of spp_sample_mfg_multi.  Because no fanout
 *     bounds the sample, the capacities of each spp_mfg decide: d_node_ids holds n_nodes_cap ids,
 *     d_indptr[h] n_nodes_cap + 1 offsets, d_src[h] n_edges_cap[h] entries.  A minibatch that
 *     would exceed them is abandoned at that hop (nothing is written out of bounds, its counts
 *     from that hop on stay 0) and the call reports SPP_E_CAPACITY when SPP_SYNC is set. */
int  spp_sample_mfg_general(spp_ctx* ctx, const spp_graph* g, const float* const* d_t,
                            const spp_sample_item* items, int32_t n_items, int32_t L, uint64_t seed,
                            uint32_t flags);

/* (f) Empirical access frequencies (Sec. 3.2, the "sim." and "oracle" caching policies): d_count[v]
 *     += 1 for every id of every list, e.g. the sampled vertex sets of the minibatches of simulated
 *     epochs ("sim.") or of the epochs being evaluated ("oracle", retroactive).  The counts are a
 *     score like any other: spp_build_vip_cache and spp_build_local_store rank them.
 *     d_count is device float32[N], not cleared by the call; counts are exact below 2^24.
 *     List j has n ids, or *d_n of them (device int64, capped at n) when d_n is given.  An id
 *     outside [0, N) is skipped; with SPP_SYNC the call then returns SPP_E_ARG after counting the
 *     others (without SPP_SYNC it goes unreported).  At most SPP_MAX_GATHER_LISTS lists. */
typedef struct {
    const int32_t* d_ids;
    int64_t        n;
    const int64_t* d_n;      /* device int64 count, or NULL */
} spp_id_list;
int  spp_access_count(spp_ctx* ctx, const spp_id_list* lists, int32_t n_lists, int64_t N, float* d_count,
                      uint32_t flags);

/* Device-time accounting.  After spp_ctx_timing(ctx, 1) every call brackets its pieces of device
 * work with events on the stream they run on (vip total and per hop, the whole sampling of a
 * batch, gather classify / hit copy / miss copy).  spp_ctx_times waits for the context's streams,
 * returns for each SPP_T_* index the summed duration in milliseconds and the number of pieces
 * since the last call, and starts a new accumulation.  spp_ctx_timing(ctx, 0) stops recording. */
enum { SPP_T_VIP_TOTAL = 0, SPP_T_VIP_HOP_FIRST = 1 /* .. +L-1 */, SPP_T_SAMPLE = 9,
       SPP_T_GATHER_HIT = 10, SPP_T_GATHER_MISS = 11, SPP_T_GATHER_CLASSIFY = 12, SPP_T_COUNT = 16 };
int  spp_ctx_timing(spp_ctx* ctx, int enable);
int  spp_ctx_times(spp_ctx* ctx, float* sum_ms /* [SPP_T_COUNT] */, int64_t* count /* [SPP_T_COUNT] */);
/*     The same with the shortest and the median piece per index (0 where there was none); any of the
 *     four arrays may be null. */
int  spp_ctx_time_stats(spp_ctx* ctx, float* sum_ms, int64_t* count, float* min_ms, float* median_ms);

/* What the part reaches by direction, measured with three plain streaming kernels of this library over
 * caller-provided device buffers of `bytes` bytes each (a multiple of 16; both 16-byte aligned): the
 * figures that the roofline fractions of Sec.-4.3-style byte-moving kernels are read against, beside the
 * published peak (which counts reads and writes together).  out_gbps[0]: a read-only pass over d_a;
 * [1]: a copy d_a -> d_b (bytes read plus bytes written); [2]: a write-only fill of d_b; each in GB/s,
 * averaged over `reps` passes (1 .. 1000) after one untimed pass.  d_b is overwritten.  Waits for
 * the context's stream. */
int  spp_stream_rates(spp_ctx* ctx, const void* d_a, void* d_b, int64_t bytes, int32_t reps, float* out_gbps /* [3] */);

/* Running sums over the calls made on this context since the last reset, kept on the device so
 * that a loop of asynchronous calls can be accounted for without a host round trip per batch:
 *   out[0] minibatches sampled, out[1] sum of |S_L|, out[2] sum of sampled edges over all hops,
 *   out[3] gather calls, out[4] rows from the local shard, out[5] rows from the cache,
 *   out[6] rows missed (neither local nor cached), out[7] local rows read from host memory,
 *   out[8] missed rows served by a copy of another row of the same call (n_miss_shared),
 *   out[9..15] unused.
 * Waits for the context's streams. */
int  spp_ctx_totals(spp_ctx* ctx, int64_t* out /* [16] */, int reset);

#ifdef __cplusplus
}
#endif
#endif /* SPP_H */
